"""GPU parity of the replica gradient path of Sec. 4.1 (per-slot weight gradients, then
add into the representative, scale, copy) against the oracle, and against the fused
per-class path of symi_expert_bwd."""
import numpy as np
import pytest
import torch

import paper_2504_19925_amd as symi
from oracle import symi_oracle as O
import harness as Hn
from tests.checks import small as _small
from harness.metrics import check_close, relerr_elem, TOL

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,it,scale", [("c1", 0, 1.0), ("c2", 1, 1.0), ("c4", 2, 0.125), ("c3", 0, 1.0)])
def test_replica_gradient_path(name, it, scale):
    c = _small(name)
    st = Hn.State(c)
    X, logits, dY = Hn.draw_inputs(c, it)
    if it > 0:
        st.hist_prev.copy_(torch.from_numpy(O.route(Hn.npf(Hn.draw_inputs(c, it - 1)[1]), c.k, True)[2]).int())
    st.place_current()
    st.forward(X, logits)
    st.backward(dY, logits)                         # fused per-class gradients in st.dW1 / st.dW2
    s, ctx = st, st.ctx
    g1 = torch.full((c.S_tot, 2 * c.f, c.d), float("nan"), dtype=torch.float32, device="cuda")
    g2 = torch.full((c.S_tot, c.d, c.f), float("nan"), dtype=torch.float32, device="cuda")
    dXp2 = torch.empty_like(s.dXp)
    symi.symi_expert_bwd_slots(ctx, s.dYp, s.Xp, s.UV, s.H, s.slot_offsets, s.first_slot, s.W1s, s.W2s,
                               dXp2, g1, g2, s.ws)
    Hn.sync()
    assert torch.equal(dXp2, s.dXp)                 # the data gradient does not depend on the variant
    # ---- per-slot gradients against the oracle
    Xn, dYn, zn = Hn.npf(X), Hn.npf(dY), Hn.npf(logits)
    W1n, W2n = Hn.npf(st.W1c), Hn.npf(st.W2c)
    o_idx, o_gate, _ = O.route(zn, c.k, True)
    o_counts, o_place, o_first = O.place(st.hist_prev.cpu().numpy(), c.S_tot)
    o_roa, _, o_off = O.dispatch(o_idx, o_counts, o_first)
    og1, og2 = O.slot_gradients(Xn, o_idx, o_gate, W1n, W2n, dYn, o_roa, o_off)
    log = {}
    check_close("dW1_slot", Hn.npf(g1), og1, c.dtype, group_axis=0, log=log)
    check_close("dW2_slot", Hn.npf(g2), og2, c.dtype, group_axis=0, log=log)
    for q in np.nonzero(np.diff(o_off) == 0)[0]:
        assert not g1[q].any() and not g2[q].any()
    # ---- the all-reduce on its own (fed the GPU's per-slot gradients): an fp32 computation
    r1 = O.replica_allreduce(Hn.npf(g1), o_first, scale)
    r2 = O.replica_allreduce(Hn.npf(g2), o_first, scale)
    symi.symi_replica_allreduce(ctx, s.first_slot, scale, g1, g2)
    Hn.sync()
    assert relerr_elem(Hn.npf(g1), r1) <= TOL["f32"] and relerr_elem(Hn.npf(g2), r2) <= TOL["f32"]
    # every replica of a class holds the same bits as its representative
    pl = torch.from_numpy(o_place).long().cuda()
    rep = st.first_slot[:-1].long()[pl]
    assert torch.equal(g1, g1[rep]) and torch.equal(g2, g2[rep])
    # ---- and the representative agrees with the fused per-class gradient
    first = st.first_slot[:-1].long()
    check_close("rep_vs_fused_dW1", Hn.npf(g1[first]), scale * Hn.npf(st.dW1).astype(np.float64), c.dtype,
                group_axis=0, log=log)
    check_close("rep_vs_fused_dW2", Hn.npf(g2[first]), scale * Hn.npf(st.dW2).astype(np.float64), c.dtype,
                group_axis=0, log=log)
    print("[err] " + " ".join(f"{k}:max={v['max']:.2e}" for k, v in log.items()), flush=True)


def test_replica_path_full_size_c2_matches_fused_path():
    """Config c2 at full size, placement mimicking the previous iteration (hot classes
    replicated over many slots): after the all-reduce every slot of a class holds the class
    gradient that the fused path computes (same products, different summation order), and
    slots without rows contributed zeros."""
    import workloads as wl
    c = wl.get_config("c2")
    st = Hn.State(c)
    X0, logits0, dY0 = Hn.draw_inputs(c, 0)
    st.place_current()
    st.forward(X0, logits0)
    st.hist_prev.copy_(st.hist)
    st.place_current()                                  # replicas proportional to iteration 0's popularity
    st.forward(X0, logits0)
    st.backward(dY0, logits0)
    s, ctx = st, st.ctx
    g1 = torch.full((c.S_tot, 2 * c.f, c.d), float("nan"), dtype=torch.float32, device="cuda")
    g2 = torch.full((c.S_tot, c.d, c.f), float("nan"), dtype=torch.float32, device="cuda")
    symi.symi_expert_bwd_slots(ctx, s.dYp, s.Xp, s.UV, s.H, s.slot_offsets, s.first_slot, s.W1s, s.W2s,
                               s.dXp, g1, g2, s.ws)
    Hn.sync()
    off = s.slot_offsets.cpu().numpy()
    assert int(s.counts.max()) > 4                      # the hot classes really are replicated
    for q in np.nonzero(np.diff(off) == 0)[0][:8]:
        assert not g1[q].any() and not g2[q].any()
    symi.symi_replica_allreduce(ctx, s.first_slot, 1.0, g1, g2)
    Hn.sync()
    pl = s.placement.long()
    for e in torch.unique(pl).tolist()[:6] + [int(s.counts.argmax())]:
        for q in torch.nonzero(pl == e).flatten().tolist()[:3]:
            a1, b1 = g1[q].double(), st.dW1[e].double()
            a2, b2 = g2[q].double(), st.dW2[e].double()
            scale1, scale2 = b1.abs().max().item() + 1e-30, b2.abs().max().item() + 1e-30
            assert (a1 - b1).abs().max().item() / scale1 <= 1e-5
            assert (a2 - b2).abs().max().item() / scale2 <= 1e-5
