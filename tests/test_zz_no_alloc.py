"""symi_dispatch_noalloc (scratch in a static device buffer, nothing allocated) against
symi_dispatch (scratch in the caller's workspace): same bits, on two calls in a row that share
the one buffer, the second with a smaller input; limits refused with an error."""
import pytest
import torch

import harness as Hn
import paper_2504_19925_amd as symi
import workloads as wl

pytestmark = pytest.mark.gpu


def _both(c, it):
    st = Hn.State(c)
    X, logits, _ = Hn.draw_inputs(c, it)
    st.hist_prev.copy_(torch.randint(0, 1000, (c.E,), dtype=torch.int32, device="cuda",
                                     generator=torch.Generator(device="cuda").manual_seed(11 + it)))
    symi.symi_place(st.ctx, st.hist_prev, st.counts, st.placement, st.first_slot)
    symi.symi_route(st.ctx, logits, st.idx, st.gate, st.hist)
    outs = []
    for noalloc in (False, True):
        bufs = [st.row_of_assign, st.assign_of_row, st.slot_offsets]
        for t in bufs:
            t.fill_(-7)
        st.Xp.fill_(float("nan"))
        if noalloc:
            symi.symi_dispatch_noalloc(st.ctx, X, st.idx, st.hist, st.counts, st.first_slot, st.row_of_assign,
                                       st.assign_of_row, st.slot_offsets, st.Xp)
        else:
            symi.symi_dispatch(st.ctx, X, st.idx, st.hist, st.counts, st.first_slot, st.row_of_assign,
                               st.assign_of_row, st.slot_offsets, st.Xp, st.ws)
        Hn.sync()
        outs.append([t.clone() for t in bufs + [st.Xp]])
    for a, b in zip(*outs):
        assert torch.equal(a, b)
    assert int(outs[1][2][-1]) == c.A                      # every assignment has a row
    assert torch.equal(outs[1][3], X[(outs[1][1] // c.k).long()])


def test_noalloc_dispatch_equals_dispatch_on_consecutive_calls():
    big = wl.scaled(wl.get_config("c4"), d=256, f=64, T=9000)          # 54 000 assignments, 53 chunks
    small = wl.scaled(wl.get_config("c2"), d=64, f=64, T=700, E=16, S_tot=24)   # then a smaller one
    for c in (big, small, wl.scaled(wl.get_config("c1"), T=300), big):
        print(f"[noalloc] {c.name} T={c.T} E={c.E} k={c.k} d={c.d} {c.dtype}", flush=True)
        _both(c, 0)


def test_noalloc_dispatch_refuses_what_does_not_fit():
    # 2^21 + 1024 assignments in 1024 classes: (2049 + 1) * 1024 * 4 bytes > 4 MiB
    c = wl.scaled(wl.get_config("c1"), dtype="bf16", T=(1 << 21) // 16 + 64, E=1024, k=16, S_tot=1024, N=1, d=8, f=8,
                  router_matmul=False)
    ctx = Hn.make_ctx(c)
    z = torch.zeros(8, dtype=torch.int32, device="cuda")
    with pytest.raises(symi.SymiError, match="static buffer"):
        symi.lib()  # loaded
        rc = symi.lib().symi_dispatch_noalloc(ctx.ptr, None, None, None, None, None, None, None, None, None, None)
        symi.binding._check(rc, "symi_dispatch_noalloc")
    timed = Hn.make_ctx(wl.scaled(wl.get_config("c1"), T=64), flags=symi.CTX_TIMING)
    rc = symi.lib().symi_dispatch_noalloc(timed.ptr, None, None, None, None, None, None, None, None, None, None)
    assert rc == -1 and "SYMI_CTX_TIMING" in symi.symi_last_error()
    del z
