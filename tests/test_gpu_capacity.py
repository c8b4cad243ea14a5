"""GPU parity of the capacity-limited dispatch (Sec. 3.4) and of the layer around it.

symi_dispatch_capacity's integers are compared bit for bit with the oracle; the layer
outputs and gradients are compared with the oracle's dropless definition evaluated with the
gates of dropped assignments set to zero (a dropped assignment contributes nothing).
"""
import numpy as np
import pytest
import torch

import paper_2504_19925_amd as symi
import workloads as wl
from oracle import symi_oracle as O
import harness as Hn
from tests.checks import small as _small
from harness.metrics import check_close

pytestmark = pytest.mark.gpu


def _run(c, capacity_factor, it=0, uniform=False):
    st = Hn.State(c)
    X, logits, dY = Hn.draw_inputs(c, it)
    zn = Hn.npf(logits)
    if not uniform and it > 0:
        # placement from the previous iteration's popularity (the paper's policy)
        st.hist_prev.copy_(torch.from_numpy(O.route(Hn.npf(Hn.draw_inputs(c, it - 1)[1]), c.k, True)[2]).int())
    st.place_current()
    cap = symi.symi_slot_capacity(st.ctx, capacity_factor)
    assert cap == O.slot_capacity(capacity_factor, c.A, c.S_tot)
    st.forward(X, logits, slot_cap=cap)
    st.backward(dY, logits)
    Hn.sync()
    o_counts, _, o_first = O.place(st.hist_prev.cpu().numpy(), c.S_tot)
    o_idx, o_gate, o_hist = O.route(zn, c.k, True)
    roa, aor, off, keep = O.dispatch_capacity(o_idx, o_counts, o_first, cap)
    return st, (X, logits, dY), (o_idx, o_gate, o_hist, o_counts, o_first), (roa, aor, off, keep), cap


@pytest.mark.parametrize("name,cf,it", [("c1", 1.0, 0), ("c2", 1.0, 0), ("c2", 1.0, 1), ("c2", 2.0, 1),
                                        ("c4", 0.5, 2), ("c5", 1.0, 0)])
def test_capacity_dispatch_and_layer_parity(name, cf, it):
    c = _small(name)
    st, (X, logits, dY), (o_idx, o_gate, o_hist, o_counts, o_first), (roa, aor, off, keep), cap = _run(c, cf, it)
    kept = int(off[-1])
    print(f"[capacity] {name} it={it} cf={cf} slot_cap={cap} survival={kept / max(c.A, 1):.4f}", flush=True)
    # ---- integers: bit exact
    assert (st.row_of_assign.cpu().numpy() == roa).all()
    assert (st.slot_offsets.cpu().numpy() == off).all()
    assert (st.assign_of_row.cpu().numpy()[:kept] == aor).all()
    assert int(np.diff(off).max(initial=0)) <= cap
    assert torch.equal(st.Xp[:kept], X[(st.assign_of_row[:kept] // c.k).long()])
    # ---- floats: the dropless definition with the dropped gates zeroed
    Xn, dYn, zn = Hn.npf(X), Hn.npf(dY), Hn.npf(logits)
    W1n, W2n = Hn.npf(st.W1c), Hn.npf(st.W2c)
    keep2 = keep.reshape(c.T, c.k)
    gate_eff = o_gate * keep2
    log = {}
    check_close("Y", Hn.npf(st.Y), O.moe_forward(Xn, o_idx, gate_eff, W1n, W2n), c.dtype, log=log)
    dX, dW1, dW2, dgate = O.moe_backward(Xn, o_idx, gate_eff, W1n, W2n, dYn)
    dgate = dgate * keep2
    check_close("dX", Hn.npf(st.dX), dX, c.dtype, log=log)
    check_close("dW1", Hn.npf(st.dW1), dW1, c.dtype, group_axis=0, log=log)
    check_close("dW2", Hn.npf(st.dW2), dW2, c.dtype, group_axis=0, log=log)
    check_close("dgate", Hn.npf(st.dgate), dgate, c.dtype, log=log)
    assert (Hn.npf(st.dgate)[~keep2] == 0).all()
    dlog = O.route_backward(zn, o_idx, o_gate, dgate, True)
    check_close("dlogits", Hn.npf(st.dlogits), dlog, c.dtype, log=log)
    # a class whose assignments were all dropped (or that had none) has zero gradient
    kept_hist = np.bincount(o_idx.ravel()[keep], minlength=c.E)
    for e in np.nonzero(kept_hist == 0)[0]:
        assert not st.dW1[e].any() and not st.dW2[e].any()


def test_huge_capacity_equals_dropless_dispatch():
    c = _small("c2")
    st, (X, logits, dY), (o_idx, o_gate, o_hist, o_counts, o_first), (roa, aor, off, keep), cap = _run(c, 1000.0, 1)
    assert keep.all()
    r0, a0, s0 = O.dispatch(o_idx, o_counts, o_first)
    assert (st.row_of_assign.cpu().numpy() == r0).all()
    assert (st.assign_of_row.cpu().numpy() == a0).all()
    assert (st.slot_offsets.cpu().numpy() == s0).all()


@pytest.mark.parametrize("name,iters", [("c2", 3), ("c4", 5)])
def test_survival_adaptive_vs_uniform_placement_full_size(name, iters):
    """The paper's central quantity at full size (integers only): survival under the
    placement that mimics the previous iteration against the static uniform placement."""
    c = wl.get_config(name)
    ctx = Hn.make_ctx(c)
    dev = "cuda"
    i32 = dict(dtype=torch.int32, device=dev)
    ws = torch.empty(symi.symi_workspace_bytes(ctx), dtype=torch.uint8, device=dev)
    X = torch.zeros(c.T, c.d, dtype=ctx.torch_dtype, device=dev)
    Xp = torch.empty(c.A, c.d, dtype=ctx.torch_dtype, device=dev)
    idx = torch.empty(c.T, c.k, **i32); gate = torch.empty(c.T, c.k, dtype=torch.float32, device=dev)
    hist = torch.empty(c.E, **i32)
    counts = torch.empty(c.E, **i32); placement = torch.empty(c.S_tot, **i32); first = torch.empty(c.E + 1, **i32)
    roa = torch.empty(c.A, **i32); aor = torch.empty(c.A, **i32); off = torch.empty(c.S_tot + 1, **i32)
    cap = symi.symi_slot_capacity(ctx, 1.0)
    prev = torch.zeros(c.E, **i32)
    for it in range(iters):
        logits = wl.make_logits(c, it).to(dev)
        symi.symi_route(ctx, logits, idx, gate, hist)
        o_idx, _, o_hist = O.route(logits.cpu().numpy(), c.k, True)
        surv = {}
        for mode, pop in (("adaptive", prev), ("uniform", torch.zeros(c.E, **i32))):
            symi.symi_place(ctx, pop, counts, placement, first)
            symi.symi_dispatch_capacity(ctx, cap, X, idx, hist, counts, first, roa, aor, off, Xp, ws)
            Hn.sync()
            oc, _, of = O.place(pop.cpu().numpy(), c.S_tot)
            o_roa, o_aor, o_off, keep = O.dispatch_capacity(o_idx, oc, of, cap)
            assert (roa.cpu().numpy() == o_roa).all() and (off.cpu().numpy() == o_off).all()
            assert (aor.cpu().numpy()[:int(o_off[-1])] == o_aor).all()
            surv[mode] = int(off[-1]) / c.A
        print(f"[survival] {name} it={it} slot_cap={cap} adaptive={surv['adaptive']:.4f} uniform={surv['uniform']:.4f}",
              flush=True)
        prev = hist.clone()
