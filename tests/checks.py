"""Checks shared by the GPU parity tests: one iteration of the HIP path (through the C ABI)
against the CPU oracle, stage by stage."""
import numpy as np
import torch

import harness as Hn
import workloads as wl
from harness.metrics import TOL, check_close, relerr_elem, relerr_l2
from oracle import symi_oracle as O


def small(name):
    """The five workload recipes at sizes the oracle finishes in seconds: several tiles, ragged
    tails, empty groups; E, k, S_tot, N and the iteration count as stated."""
    c = wl.get_config(name)
    if name == "c1":
        return c                                                     # full size
    if name == "c2":
        return wl.scaled(c, d=256, f=384, T=1500)                    # ragged rows, f = 3 tiles
    if name == "c3":
        return wl.scaled(c, d=512, f=1000, T=2100)                   # f not a tile multiple
    if name == "c4":
        return wl.scaled(c, d=192, f=352, T=1111)                    # top-6, 128 slots
    if name == "c5":
        return wl.scaled(c, d=256, f=136, T=3001)                    # top-8, 256 slots
    raise KeyError(name)


def check_iteration(st: Hn.State, X, logits, dY, hp_kw=None, check_float=True, chained=False,
                    log=None):
    """One full iteration on the GPU, every stage compared with the oracle.

    chained=False: the slots are materialised from the state's (never updated) class weights
    before the forward, the state's own optimizer partition steps.
    chained=True (a state holding all N partitions): the forward consumes the slots as the
    previous iteration's symi_adam_to_replicas calls left them under the placement that
    st.advance() moved into place; only the very first iteration materialises them.  The class
    weights the oracle uses are then read back from the slots (they are the GPU's own, bf16- or
    fp32-valued, weights), every replica of a class must hold the same bits, and after the
    optimizer every slot of the next placement must equal the cast of its class's master
    weights over the whole parameter vector."""
    c, ctx = st.c, st.ctx
    hist_prev = st.hist_prev.cpu().numpy()
    first = not (chained and getattr(st, "_chain_started", False))
    if first:
        st.place_current()
        st._chain_started = chained
    if chained:
        rep = st.first_slot[:-1].long()[st.placement.long()]      # slot -> first slot of its class
        assert torch.equal(st.W1s, st.W1s[rep]) and torch.equal(st.W2s, st.W2s[rep])
        W1g, W2g = st.W1s[st.first_slot[:-1].long()], st.W2s[st.first_slot[:-1].long()]
    else:
        W1g, W2g = st.W1c, st.W2c
    st.forward(X, logits)
    if st.active_grads:      # the *_active pair must neither write nor read these
        st.dW1.fill_(float("nan"))
        st.dW2.fill_(float("nan"))
    st.backward(dY, logits)
    adam, hp = Hn.make_adam(**(hp_kw or {}))
    state0 = {n: (Hn.npf(w), Hn.npf(m), Hn.npf(v)) for n, (_, w, m, v) in st.opt.items()}
    W1s0, W2s0 = Hn.npf(st.W1s).copy(), Hn.npf(st.W2s).copy()
    st.optimizer(adam)
    Hn.sync()

    Xn, zn, dYn = Hn.npf(X), Hn.npf(logits), Hn.npf(dY)
    # ---- integers: bit exact
    o_counts, o_place, o_first = O.place(hist_prev, c.S_tot)
    assert (st.counts.cpu().numpy() == o_counts).all()
    assert (st.placement.cpu().numpy() == o_place).all()
    assert (st.first_slot.cpu().numpy() == o_first).all()
    o_idx, o_gate, o_hist = O.route(zn, c.k, bool(ctx.renorm))
    assert (st.idx.cpu().numpy() == o_idx).all()
    assert (st.hist.cpu().numpy() == o_hist).all()
    assert o_hist.sum() == c.A
    o_roa, o_aor, o_off = O.dispatch(o_idx, o_counts, o_first)
    assert (st.row_of_assign.cpu().numpy() == o_roa).all()
    assert (st.assign_of_row.cpu().numpy() == o_aor).all()
    assert (st.slot_offsets.cpu().numpy() == o_off).all()
    n_counts, n_place, n_first = O.place(o_hist, c.S_tot)
    assert (st.counts_next.cpu().numpy() == n_counts).all()
    assert (st.placement_next.cpu().numpy() == n_place).all()
    assert (st.first_slot_next.cpu().numpy() == n_first).all()
    # the gather is a copy: bit exact
    if c.A:
        assert torch.equal(st.Xp, X[(st.assign_of_row // c.k).long()])
    if not check_float:
        return
    # ---- floats.  Axis whose outputs share their error scale (floor of the element-wise
    # measure, harness/metrics.py): a token's row of Y and dX, the f hidden units of an input
    # column in each half of dW1 [E,2,f,d], the d outputs of a hidden unit in dW2 [E,d,f].
    log = {} if log is None else log
    assert relerr_elem(Hn.npf(st.gate), o_gate) <= TOL["f32"]
    W1n, W2n = Hn.npf(W1g), Hn.npf(W2g)
    Y = O.moe_forward(Xn, o_idx, o_gate, W1n, W2n)
    check_close("Y", Hn.npf(st.Y), Y, c.dtype, log=log, iid_axis=1, K=c.f)
    dX, dW1, dW2, dgate = O.moe_backward(Xn, o_idx, o_gate, W1n, W2n, dYn)
    dlog = O.route_backward(zn, o_idx, o_gate, dgate, bool(ctx.renorm))
    check_close("dX", Hn.npf(st.dX), dX, c.dtype, log=log, iid_axis=1, K=2 * c.f)
    gW1, gW2 = Hn.npf(st.dW1), Hn.npf(st.dW2)
    empty = np.nonzero(o_hist == 0)[0]
    if st.active_grads:
        # gradients of classes without rows: left as they were, and zero for the optimizer
        assert np.isnan(gW1[empty]).all() and np.isnan(gW2[empty]).all()
        gW1[empty] = 0.0
        gW2[empty] = 0.0
    kmax = int(o_hist.max()) if c.E else 1
    half = (c.E, 2, c.f, c.d)
    check_close("dW1", gW1.reshape(half), dW1.reshape(half), c.dtype, group_axis=0, log=log, iid_axis=2, K=kmax)   # per class
    check_close("dW2", gW2, dW2, c.dtype, group_axis=0, log=log, iid_axis=1, K=kmax)
    check_close("dgate", Hn.npf(st.dgate), dgate, c.dtype, log=log)
    check_close("dlogits", Hn.npf(st.dlogits), dlog, c.dtype, log=log)
    print("[err] " + " ".join(
        f"{k}:max={v['max']:.2e},l2={v['l2']:.2e},elem={v['elem']:.2e}" +
        (f",axis={v['axis']:.2e}/{v['axis_bound']:.2e}" if "axis" in v else "")
        for k, v in log.items()), flush=True)
    # the router backward on its own (fed the same dgate) is an fp32 computation
    dlog_iso = O.route_backward(zn, o_idx, Hn.npf(st.gate), Hn.npf(st.dgate), bool(ctx.renorm))
    assert relerr_elem(Hn.npf(st.dlogits), dlog_iso) <= TOL["f32"]
    # classes without rows have exactly zero gradient
    for e in empty:
        assert not gW1[e].any() and not gW2[e].any()
    # ---- Adam on every held partition, fed the GPU's own gradients (stage isolated)
    per = c.P_e // c.N
    slots = torch.cat([st.W1s.reshape(c.S_tot, -1), st.W2s.reshape(c.S_tot, -1)], 1)
    sl = Hn.npf(slots)
    before = np.concatenate([W1s0.reshape(c.S_tot, -1), W2s0.reshape(c.S_tot, -1)], 1)
    W1s_o, W2s_o = W1s0.copy(), W2s0.copy()
    written = np.zeros(c.P_e, dtype=bool)
    for n, (_, w_g, m_g, v_g) in st.opt.items():
        master0, m0, v0 = state0[n]
        w2, m2, v2 = O.adam_to_replicas(gW1, gW2, master0, m0, v0, n_place, c.N, n, hp,
                                        c.dtype == "bf16", W1s_o, W2s_o)
        assert relerr_elem(Hn.npf(w_g), w2) <= TOL["adam"]
        assert relerr_elem(Hn.npf(m_g), m2) <= TOL["adam"]
        assert relerr_elem(Hn.npf(v_g), v2) <= TOL["adam"]
        # slots: exactly the rounding of the GPU's own fresh master weights on the partition's
        # range of every slot of the NEXT placement
        lo = n * per
        want = w_g[st.placement_next.long()].to(st.W1s.dtype)
        assert torch.equal(slots[:, lo:lo + per], want)
        written[lo:lo + per] = True
    # ... untouched elsewhere
    assert (sl[:, ~written] == before[:, ~written]).all()
    if chained:
        assert written.all()
    # and close to the oracle's slots: the two master weights differ by at most the Adam
    # tolerance (relative to max(|w|, rms), which matters for weights the step moves to ~0) and
    # their bf16 roundings by one more ulp where that difference straddles a rounding boundary
    so = np.concatenate([W1s_o.reshape(c.S_tot, -1), W2s_o.reshape(c.S_tot, -1)], 1)
    if c.dtype == "bf16":
        rms = float(np.sqrt(np.mean(so[:, written] ** 2))) if per else 0.0
        assert (np.abs(sl - so) <= 2.0 ** -7 * np.abs(so) + 2 * TOL["adam"] * rms + 1e-30).all()
    else:
        assert relerr_elem(sl, so) <= TOL["adam"]


class OracleChain:
    """The oracle on its own from the first iteration on: its own class weights, moments and
    placements, never fed anything the GPU computed.  After the last iteration the distance of
    the GPU's master weights and moments from this chain is the end-to-end drift (reported; the
    asserted tolerances are the stage-isolated ones)."""

    def __init__(self, c, W1c, W2c):
        self.c = c
        E = c.E
        self.w = np.concatenate([Hn.npf(W1c).reshape(E, -1), Hn.npf(W2c).reshape(E, -1)], 1).astype(np.float64)
        self.m = np.zeros_like(self.w)
        self.v = np.zeros_like(self.w)

    def class_weights(self):
        c = self.c
        w = self.w.astype(np.float32)
        if c.dtype == "bf16":
            w = O.round_to_bf16(w)
        n1 = 2 * c.f * c.d
        return w[:, :n1].reshape(c.E, 2 * c.f, c.d), w[:, n1:].reshape(c.E, c.d, c.f)

    def step(self, X, logits, dY, hp):
        c = self.c
        Xn, zn, dYn = Hn.npf(X), Hn.npf(logits), Hn.npf(dY)
        idx, gate, _ = O.route(zn, c.k, True)
        W1, W2 = self.class_weights()
        _, dW1, dW2, _ = O.moe_backward(Xn, idx, gate, W1, W2, dYn)
        g = np.concatenate([dW1.reshape(c.E, -1), dW2.reshape(c.E, -1)], 1)
        self.w, self.m, self.v = O.adam_step(self.w, self.m, self.v, g, hp["lr"], hp["beta1"], hp["beta2"],
                                             hp["eps"], hp["weight_decay"], hp["grad_scale"], hp["step"])

    def drift(self, st):
        """Distance of the GPU's (master, m, v), all partitions side by side, to the chain's:
        relative L2 and the element-wise measure (floor: rms).  Adam divides by the root of the
        second moment, so an element whose gradient is within the arithmetic's noise of zero
        moves by a full +-lr per step in a direction the noise decides: a few such elements
        make the element-wise distance large after some steps while the L2 distance stays
        small."""
        per = self.c.P_e // self.c.N
        out = {}
        for name, i, mine in (("master", 1, self.w), ("m", 2, self.m), ("v", 3, self.v)):
            got = np.concatenate([Hn.npf(st.opt[n][i]) for n in range(self.c.N)], 1)
            assert got.shape[1] == per * self.c.N
            out[name + "_l2"] = relerr_l2(got, mine)
            out[name + "_elem"] = relerr_elem(got, mine)
        return out


def stratified_tokens(slot_offsets, assign_of_row, k, T, rng, n_random=48, max_edges=256, tile=256):
    """Tokens for a sampled float check that are guaranteed to exercise the tile structure of
    the grouped GEMM: for every slot that holds rows the token of its first and of its last
    row, and the tokens of the two rows on either side of m-tile edges inside slots (all such
    edges if there are at most `max_edges`, else that many drawn at random), topped up with
    `n_random` tokens drawn uniformly.  Returns sorted unique token ids and the number of rows
    that were picked for structural reasons."""
    off = np.asarray(slot_offsets, dtype=np.int64)
    rows, edges = [], []
    for q in range(len(off) - 1):
        a, b = int(off[q]), int(off[q + 1])
        if b == a:
            continue
        rows += [a, b - 1]
        edges += [(r - 1, r) for r in range(a + tile, b, tile)]
    if len(edges) > max_edges:
        edges = [edges[i] for i in rng.choice(len(edges), size=max_edges, replace=False)]
    for lo, hi in edges:
        rows += [lo, hi]
    rows = np.unique(np.asarray(rows, dtype=np.int64))
    toks = np.asarray(assign_of_row)[rows] // k if rows.size else np.zeros(0, dtype=np.int64)
    extra = rng.choice(T, size=min(n_random, T), replace=False)
    return np.unique(np.concatenate([toks, extra]).astype(np.int64)), int(rows.size)


def adam_check_threaded(got, state0, g, hp, tol, slab=4, workers=8):
    """Oracle Adam step on (master, m, v) = state0 with gradient g (all [E, n] numpy fp32),
    compared with the GPU's `got` triple at `tol` (relerr_elem per slab of classes).  Slabs run
    on a thread pool: numpy releases the interpreter lock inside its array loops."""
    from concurrent.futures import ThreadPoolExecutor
    E = g.shape[0]

    def one(e0):
        sl = slice(e0, min(e0 + slab, E))
        w2, m2, v2 = O.adam_step(state0[0][sl], state0[1][sl], state0[2][sl], g[sl], hp["lr"], hp["beta1"],
                                 hp["beta2"], hp["eps"], hp["weight_decay"], hp["grad_scale"], hp["step"])
        return max(relerr_elem(got[0][sl], w2), relerr_elem(got[1][sl], m2), relerr_elem(got[2][sl], v2))

    with ThreadPoolExecutor(max_workers=workers) as ex:
        worst = max(ex.map(one, range(0, E, slab)))
    assert worst <= tol, f"Adam state: element-wise error {worst:.3e} > {tol:g}"
    return worst
