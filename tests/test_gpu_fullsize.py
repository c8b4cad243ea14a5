"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.

The oracle cannot run a whole full-size layer in seconds, so floating-point outputs are
checked on samples it can compute one by one, using two facts of the definition:
  * tokens are independent: Y[t], dX[t], dgate[t], dlogits[t] of a sampled token equal the
    oracle's result on the batch made of the sampled tokens alone;
  * hidden units are independent in the weight gradient: dW restricted to a few hidden
    units equals the gradient of the FFN that keeps only those units (pinned on the CPU in
    test_oracle_layer_adam.py), so the oracle runs ALL tokens through 4..8-unit experts.
Integer outputs are compared in full, bit for bit; the Adam state of the whole shard is
compared in full."""
import numpy as np
import pytest
import torch

import harness as Hn
import paper_2504_19925_amd as symi
import workloads as wl
from harness.metrics import TOL, check_close, relerr_elem
from oracle import symi_oracle as O
from tests.checks import adam_check_threaded, stratified_tokens

pytestmark = pytest.mark.gpu

N_RANDOM = 48      # uniformly drawn tokens on top of the structural sample
N_UNITS = {"c2": 8, "c3": 8, "c4": 6, "c5": 4}


def _shard_gradient(st, n):
    """The flat gradient range [E, P_e/N] of optimizer partition n, cut from dW1 | dW2."""
    c = st.c
    per = c.P_e // c.N
    lo, n1 = n * per, 2 * c.f * c.d
    parts = []
    if lo < n1:
        parts.append(st.dW1.reshape(c.E, -1)[:, lo:min(lo + per, n1)])
    if lo + per > n1:
        parts.append(st.dW2.reshape(c.E, -1)[:, max(lo - n1, 0):lo + per - n1])
    g = torch.cat(parts, 1)
    assert g.shape[1] == per
    return g


@pytest.mark.parametrize("name", ["c2", "c3", "c4", "c5"])
@pytest.mark.timeout(900)
def test_fullsize_parity(name):
    """Full size, the launch configuration bench.py times.  c2 and c4 walk their whole schedule
    (10 and 20 iterations) as one chain: all N optimizer partitions step, iteration t+1
    dispatches with the placement made from iteration t's popularity and computes on the slots
    iteration t's optimizer wrote.  Every iteration: all integer outputs in full and the Adam
    state of one whole partition against the oracle.  Last iteration: floats on a sample that
    covers every slot's first and last row and its m-tile edges, and on sampled hidden units
    of every class gradient.  c3 and c5 state one iteration; their placement mimics the batch's
    own popularity so that hot classes own many replicas."""
    import time
    c = wl.get_config(name)
    print(f"[fullsize] {name}: T={c.T} E={c.E} k={c.k} d={c.d} f={c.f} S_tot={c.S_tot} N={c.N} "
          f"iterations={c.iters}", flush=True)
    rng = np.random.default_rng(1234 + c.seed)
    chain = c.iters > 1
    shard = c.N - 1
    st = Hn.State(c, shard=shard, all_shards=chain)
    ctx = st.ctx
    per = c.P_e // c.N
    lo = shard * per
    n1 = 2 * c.f * c.d
    for it in range(c.iters):
        t_start = time.perf_counter()
        last = it == c.iters - 1
        X, logits, dY = Hn.draw_inputs(c, it)
        if not chain:
            # placement that mimics this very popularity: hot classes own many replicas
            symi.symi_route(ctx, logits, st.idx, st.gate, st.hist)
            st.hist_prev.copy_(st.hist)
            st.m.normal_(generator=torch.Generator(device="cuda").manual_seed(7)).mul_(1e-3)
            st.v.uniform_(1e-8, 1e-6, generator=torch.Generator(device="cuda").manual_seed(8))
        hist_prev = st.hist_prev.cpu().numpy()
        if it == 0:
            st.place_current()           # c2/c4: no history yet -> uniform placement
        else:
            # every replica of a class holds the same bits, written by the N partitions
            rep = st.first_slot[:-1].long()[st.placement.long()]
            for q0 in range(0, c.S_tot, 16):
                qs = slice(q0, min(q0 + 16, c.S_tot))
                assert torch.equal(st.W1s[qs], st.W1s[rep[qs]]) and torch.equal(st.W2s[qs], st.W2s[rep[qs]])
        W1g = st.W1s[st.first_slot[:-1].long()] if chain and last else st.W1c   # the GPU's current
        W2g = st.W2s[st.first_slot[:-1].long()] if chain and last else st.W2c   # class weights
        st.forward(X, logits)
        st.backward(dY, logits)
        adam, hp = Hn.make_adam(step=it + 1 if chain else 3, weight_decay=0.01)
        state0 = [t.clone() for t in (st.master, st.m, st.v)]
        st.optimizer(adam)
        Hn.sync()

        # ---- integers, in full
        zn = Hn.npf(logits)
        o_counts, o_place, o_first = O.place(hist_prev, c.S_tot)
        o_idx, o_gate, o_hist = O.route(zn, c.k, True)
        o_roa, o_aor, o_off = O.dispatch(o_idx, o_counts, o_first)
        n_counts, n_place, n_first = O.place(o_hist, c.S_tot)
        for got, want in [(st.counts, o_counts), (st.placement, o_place), (st.first_slot, o_first),
                          (st.idx, o_idx), (st.hist, o_hist), (st.row_of_assign, o_roa),
                          (st.assign_of_row, o_aor), (st.slot_offsets, o_off),
                          (st.counts_next, n_counts), (st.placement_next, n_place),
                          (st.first_slot_next, n_first)]:
            assert (got.cpu().numpy() == want).all()
        assert torch.equal(st.Xp, X[(st.assign_of_row // c.k).long()])
        assert relerr_elem(Hn.npf(st.gate), o_gate) <= TOL["f32"]

        # ---- Adam on the whole partition, fed the GPU's own gradients; replica slots
        worst = adam_check_threaded([Hn.npf(t) for t in (st.master, st.m, st.v)], [Hn.npf(t) for t in state0],
                                    Hn.npf(_shard_gradient(st, shard)), hp, TOL["adam"])
        pl = st.placement_next.long()
        for n, (_, w_n, _, _) in st.opt.items():
            a = n * per
            for q0 in range(0, c.S_tot, 32):
                qs = slice(q0, min(q0 + 32, c.S_tot))
                slots = torch.cat([st.W1s[qs].reshape(-1, n1), st.W2s[qs].reshape(-1, c.d * c.f)], 1)[:, a:a + per]
                assert torch.equal(slots, w_n[pl[qs]].to(st.W1s.dtype))
        print(f"[fullsize] {name} iteration {it}: integers, Adam state of partition {shard} ({worst:.1e}) and "
              f"slots ok; slot rows min/max = {np.diff(o_off).min()}/{np.diff(o_off).max()}, replicas max = "
              f"{o_counts.max()}; {time.perf_counter() - t_start:.1f} s", flush=True)
        if not last:
            st.hist_prev.copy_(st.hist)
            st.advance()
            continue

        # ---- sampled tokens: Y, dX, dgate, dlogits
        ts, n_struct = stratified_tokens(o_off, o_aor, c.k, c.T, rng, n_random=N_RANDOM)
        tt = torch.tensor(ts, device="cuda")
        W1L, W2L = Hn.LazyWeights(W1g), Hn.LazyWeights(W2g)
        Xs, dYs, zs = Hn.npf(X[tt]), Hn.npf(dY[tt]), zn[ts]
        Ys = O.moe_forward(Xs, o_idx[ts], o_gate[ts], W1L, W2L)
        dXs, _, _, dgs = O.moe_backward(Xs, o_idx[ts], o_gate[ts], W1L, W2L, dYs)
        dls = O.route_backward(zs, o_idx[ts], o_gate[ts], dgs, True)
        log = {}
        check_close("Y", Hn.npf(st.Y[tt]), Ys, c.dtype, log=log, iid_axis=1, K=c.f)
        check_close("dX", Hn.npf(st.dX[tt]), dXs, c.dtype, log=log, iid_axis=1, K=2 * c.f)
        check_close("dgate", Hn.npf(st.dgate[tt]), dgs, c.dtype, log=log)
        check_close("dlogits", Hn.npf(st.dlogits[tt]), dls, c.dtype, log=log)
        print(f"[fullsize] {len(ts)} tokens ({n_struct} rows at slot ends and m-tile edges) "
              + " ".join(f"{k}:max={v['max']:.2e},l2={v['l2']:.2e}" + (f",axis={v['axis']:.2e}" if "axis" in v else "")
                         for k, v in log.items()) + f"; {time.perf_counter() - t_start:.1f} s", flush=True)

        # ---- sampled hidden units: dW1 rows (gate and up) and dW2 columns of every class
        hs = np.sort(rng.choice(c.f, size=N_UNITS[name], replace=False))
        hcat = np.concatenate([hs, c.f + hs])
        W1S = Hn.LazyWeights(W1g, rows=torch.tensor(hcat, device="cuda"))
        W2S = Hn.LazyWeights(W2g, cols=torch.tensor(hs, device="cuda"))
        _, dW1s, dW2s, _ = O.moe_backward(Hn.npf(X), o_idx, o_gate, W1S, W2S, Hn.npf(dY))
        g1 = Hn.npf(st.dW1[:, torch.tensor(hcat, device="cuda"), :])
        g2 = Hn.npf(st.dW2[:, :, torch.tensor(hs, device="cuda")])
        log = {}
        kmax = int(o_hist.max())
        # the sampled hidden units are too few for a steady rms along their own axis: the rms of
        # a unit's row over all d inputs backs the floor up
        half = (c.E, 2, len(hs), c.d)
        check_close("dW1", g1.reshape(half), dW1s.reshape(half), c.dtype, group_axis=0, log=log, iid_axis=(2, 3), K=kmax)
        check_close("dW2", g2, dW2s, c.dtype, group_axis=0, log=log, iid_axis=1, K=kmax)
        print("[fullsize] units " + " ".join(f"{k}:max={v['max']:.2e},l2={v['l2']:.2e},axis={v['axis']:.2e}"
                                             for k, v in log.items()) + f"; {time.perf_counter() - t_start:.1f} s",
              flush=True)
        for e in np.nonzero(o_hist == 0)[0][:4]:
            assert not st.dW1[e].any() and not st.dW2[e].any()


@pytest.mark.timeout(600)
def test_sliced_tail_tiles_against_the_oracle():
    """On c2 the two narrow products (Yp, dXp) are 300 tiles: the last round's 44 tiles have
    their reduction cut into slices that a second kernel adds up.  Tokens whose rows lie in
    those tiles are checked against the oracle; the sliced result is reproducible bit for bit
    and within one bf16 rounding of the unsliced one (up to reordering noise where a sum cancels)."""
    c = wl.get_config("c2")
    st = Hn.State(c, shard=0)
    X, logits, dY = Hn.draw_inputs(c, 0)
    st.place_current()
    st.forward(X, logits)
    st.backward(dY, logits)
    Hn.sync()
    # the library's slicing rule, restated on the host
    so = st.slot_offsets.cpu().numpy()
    mt_rows = [(r, min(r + 256, so[q + 1])) for q in range(c.S_tot) for r in range(so[q], so[q + 1], 256)]
    cus = min(torch.cuda.get_device_properties(0).multi_processor_count, 256)
    ntx = -(-c.d // 256)
    n_tiles = len(mt_rows) * ntx
    rem = n_tiles % cus
    assert 0 < rem <= cus // 2, (n_tiles, cus)
    for K in (c.f, 2 * c.f):
        assert min(cus // rem, 8, -(-K // 64) // 16) >= 2
    first_sliced_mt = -(-(n_tiles - rem) // ntx)        # m-tiles all of whose tiles are sliced
    rows = np.concatenate([np.arange(a, b) for a, b in mt_rows[first_sliced_mt:]])
    assert len(rows) > 0
    rng = np.random.default_rng(99)
    pick = rng.choice(rows, size=min(40, len(rows)), replace=False)
    toks = np.unique(st.assign_of_row.cpu().numpy()[pick] // c.k)
    tt = torch.tensor(toks, device="cuda")
    o_idx, o_gate, _ = O.route(Hn.npf(logits[tt]), c.k, True)
    W1L, W2L = Hn.LazyWeights(st.W1c), Hn.LazyWeights(st.W2c)
    Ys = O.moe_forward(Hn.npf(X[tt]), o_idx, o_gate, W1L, W2L)
    dXs, _, _, _ = O.moe_backward(Hn.npf(X[tt]), o_idx, o_gate, W1L, W2L, Hn.npf(dY[tt]))
    check_close("Y", Hn.npf(st.Y[tt]), Ys, c.dtype)
    check_close("dX", Hn.npf(st.dX[tt]), dXs, c.dtype)
    # reproducible, and one rounding away from the uncut reduction at most
    Yp1, dXp1 = st.Yp.clone(), st.dXp.clone()
    st.forward(X, logits)
    st.backward(dY, logits)
    Hn.sync()
    assert torch.equal(st.Yp, Yp1) and torch.equal(st.dXp, dXp1)
    whole = symi.symi_create(st.cfg, symi.CTX_NO_SLICING)      # same buffers, reductions left whole
    st.ctx, sliced = whole, st.ctx
    st.forward(X, logits)
    st.backward(dY, logits)
    Hn.sync()
    st.ctx = sliced
    rr = torch.tensor(rows, device="cuda")
    other = torch.zeros(c.A, dtype=torch.bool, device="cuda")
    other[:mt_rows[(n_tiles - rem) // ntx][0]] = True      # rows of m-tiles with no sliced tile
    assert torch.equal(st.Yp[other], Yp1[other]) and torch.equal(st.dXp[other], dXp1[other])
    for a, b in ((st.Yp[rr], Yp1[rr]), (st.dXp[rr], dXp1[rr])):
        a, b = a.float(), b.float()
        # one bf16 rounding of the value, or (where the sum cancels) of the fp32 reordering noise
        assert ((a - b).abs() <= 2.0 ** -7 * b.abs() + 2.0 ** -12 * b.abs().max()).all()
        assert not torch.equal(a, b)        # the slices really were summed in another order
