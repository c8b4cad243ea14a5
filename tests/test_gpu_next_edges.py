"""Edge cases of the entry points around the core path: smallest shapes, an empty batch,
capacity of one row per slot, class counts that are no multiple of anything, slots without
rows.  Every case is checked against the oracle like the regular-size tests."""
import numpy as np
import pytest
import torch

import paper_2504_19925_amd as symi
import workloads as wl
from oracle import symi_oracle as O
import harness as Hn
from harness.metrics import check_close, relerr_elem, TOL

pytestmark = pytest.mark.gpu


def _cases(dtype):
    base = wl.scaled(wl.get_config("c1"), dtype=dtype)
    return [
        wl.scaled(base, T=1, E=1, k=1, S_tot=1, N=1, d=8, f=8),
        wl.scaled(base, T=5, E=4, k=4, S_tot=4, N=2, d=16, f=24),
        wl.scaled(base, T=130, E=3, k=1, S_tot=64, N=4, d=40, f=72),        # most slots empty
        wl.scaled(base, T=257, E=23, k=2, S_tot=46, N=2, d=72, f=200),      # E odd: scalar router stores
        wl.scaled(base, T=0, E=8, k=2, S_tot=16, N=4, d=128, f=256),        # empty batch
        wl.scaled(base, T=77, E=16, k=3, S_tot=16, N=2, d=24, f=40),        # one partial router row block and column tile
        wl.scaled(base, T=1300, E=8, k=2, S_tot=8, N=2, d=136, f=16),       # three router chunks, ragged last block, 8 columns in the second tile
        wl.scaled(base, T=700, E=130, k=5, S_tot=260, N=2, d=64, f=64, router_matmul=False,
                  bias="zipf", zipf_s=1.2),                                  # E > 128: two router column tiles
    ]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_router_capacity_and_replica_path_on_edge_shapes(dtype):
    for c in _cases(dtype):
        print(f"[edge] {c}", flush=True)
        st = Hn.State(c)
        s, ctx = st, st.ctx
        X, _, dY = Hn.draw_inputs(c, 0)
        Wr, b = wl.make_router(c, 0, "cuda")
        logits = torch.zeros(c.T, c.E, dtype=torch.float32, device="cuda")
        symi.symi_router_fwd(ctx, X, Wr, b, logits)
        Hn.sync()
        Xn, Wn, bn, dYn = Hn.npf(X), Hn.npf(Wr), Hn.npf(b), Hn.npf(dY)
        if c.T:
            check_close("logits", Hn.npf(logits), O.router_forward(Xn, Wn, bn), c.dtype)
        zn = Hn.npf(logits)
        # ---- capacity of ONE row per slot, then the per-slot gradient path on the kept rows
        st.place_current()
        st.forward(X, logits, slot_cap=1)
        symi.symi_combine_bwd(ctx, dY, s.Yp, s.row_of_assign, s.gate, s.dYp, s.dgate)
        g1 = torch.full((c.S_tot, 2 * c.f, c.d), float("nan"), dtype=torch.float32, device="cuda")
        g2 = torch.full((c.S_tot, c.d, c.f), float("nan"), dtype=torch.float32, device="cuda")
        symi.symi_expert_bwd_slots(ctx, s.dYp, s.Xp, s.UV, s.H, s.slot_offsets, s.first_slot, s.W1s, s.W2s,
                                   s.dXp, g1, g2, s.ws)
        symi.symi_dispatch_bwd(ctx, s.dXp, s.row_of_assign, s.dX)
        symi.symi_route_bwd(ctx, logits, s.idx, s.gate, s.dgate, s.dlogits)
        dWr = torch.empty(c.E, c.d, dtype=torch.float32, device="cuda")
        db = torch.empty(c.E, dtype=torch.float32, device="cuda")
        symi.symi_router_bwd(ctx, X, Wr, s.dlogits, dWr, db, s.dX, s.ws)
        Hn.sync()
        o_idx, o_gate, _ = O.route(zn, c.k, True)
        o_counts, o_place, o_first = O.place(np.zeros(c.E, dtype=np.int64), c.S_tot)
        roa, aor, off, keep = O.dispatch_capacity(o_idx, o_counts, o_first, 1)
        kept = int(off[-1])
        assert (s.row_of_assign.cpu().numpy() == roa).all()
        assert (s.slot_offsets.cpu().numpy() == off).all() and int(np.diff(off).max(initial=0)) <= 1
        assert (s.assign_of_row.cpu().numpy()[:kept] == aor).all()
        keep2 = keep.reshape(c.T, c.k)
        gate_eff = o_gate * keep2
        W1n, W2n = Hn.npf(st.W1c), Hn.npf(st.W2c)
        if c.T:
            check_close("Y", Hn.npf(s.Y), O.moe_forward(Xn, o_idx, gate_eff, W1n, W2n), c.dtype)
        og1, og2 = O.slot_gradients(Xn, o_idx, gate_eff, W1n, W2n, dYn, roa, off)
        check_close("dW1_slot", Hn.npf(g1), og1, c.dtype, group_axis=0)
        check_close("dW2_slot", Hn.npf(g2), og2, c.dtype, group_axis=0)
        for q in np.nonzero(np.diff(off) == 0)[0]:
            assert not g1[q].any() and not g2[q].any()
        dX_e, _, _, dgate = O.moe_backward(Xn, o_idx, gate_eff, W1n, W2n, dYn)
        dlog = O.route_backward(zn, o_idx, o_gate, dgate * keep2, True)
        o_dWr, o_db, o_dXr = O.router_backward(Xn, Wn, dlog)
        if c.T:
            check_close("dX_total", Hn.npf(s.dX), dX_e + o_dXr, c.dtype)
            check_close("dWr", Hn.npf(dWr), o_dWr, c.dtype)
            # stage-isolated: the library's own dlogits through the oracle's router backward
            i_dWr, i_db, _ = O.router_backward(Xn, Wn, Hn.npf(s.dlogits))
            check_close("dWr_isolated", Hn.npf(dWr), i_dWr, c.dtype)
            check_close("db_isolated", Hn.npf(db), i_db, "f32")
        else:
            assert not dWr.any() and not db.any()
        # ---- the all-reduce over the replicas, average over the class's replicas
        r1 = O.replica_allreduce(Hn.npf(g1), o_first, 0.5)
        symi.symi_replica_allreduce(ctx, s.first_slot, 0.5, g1, g2)
        Hn.sync()
        assert relerr_elem(Hn.npf(g1), r1) <= TOL["f32"]
