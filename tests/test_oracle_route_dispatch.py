"""Pins for the oracle's routing (Sec. 2.1, Sec. 3.2 step 1) and dispatch (step 2)."""
import numpy as np
import scipy.special
import torch

from oracle import symi_oracle as O


def _topk_brute(row, k):
    return sorted(range(len(row)), key=lambda e: (-float(row[e]), e))[:k]


def test_topk_matches_brute_force_and_tie_rule(rng):
    for T, E, k in [(1, 1, 1), (5, 3, 3), (64, 8, 2), (200, 64, 6), (50, 128, 8)]:
        z = rng.standard_normal((T, E)).astype(np.float32)
        # plant ties: quantise some rows so many logits coincide
        z[::3] = np.round(z[::3] * 2) / 2
        z[1::7] = 0.25
        idx, gate, hist = O.route(z, k)
        for t in range(T):
            assert idx[t].tolist() == _topk_brute(z[t], k)
        assert hist.sum() == T * k
        assert hist.tolist() == [int((idx == e).sum()) for e in range(E)]


def test_all_equal_row_picks_lowest_indices():
    idx, gate, hist = O.route(np.zeros((3, 8), np.float32), 3)
    assert idx.tolist() == [[0, 1, 2]] * 3
    np.testing.assert_allclose(gate, 1.0 / 3.0)


def test_gate_is_softmax_then_topk_then_renorm(rng):
    z = rng.standard_normal((40, 16)).astype(np.float32) * 3
    idx, gate, _ = O.route(z, 4, renorm=False)
    p = scipy.special.softmax(z.astype(np.float64), axis=1)        # library routine
    np.testing.assert_allclose(gate, np.take_along_axis(p, idx.astype(np.int64), 1), rtol=1e-13)
    idx2, gate2, _ = O.route(z, 4, renorm=True)
    assert (idx2 == idx).all()
    np.testing.assert_allclose(gate2.sum(1), 1.0, rtol=1e-13)
    np.testing.assert_allclose(gate2 * gate.sum(1, keepdims=True), gate, rtol=1e-13)
    assert (np.diff(gate2, axis=1) <= 0).all()                     # descending score


def test_route_backward_against_autograd_and_sum_rule(rng):
    for renorm in (True, False):
        z = rng.standard_normal((30, 12)) * 2
        idx, gate, _ = O.route(z, 3, renorm)
        dgate = rng.standard_normal(gate.shape)
        dl = O.route_backward(z, idx, gate, dgate, renorm)
        zt = torch.tensor(z, dtype=torch.float64, requires_grad=True)
        p = torch.softmax(zt, dim=1)
        g = torch.gather(p, 1, torch.tensor(idx, dtype=torch.int64))
        if renorm:
            g = g / g.sum(1, keepdim=True)
        (g * torch.tensor(dgate)).sum().backward()
        np.testing.assert_allclose(dl, zt.grad.numpy(), rtol=1e-10, atol=1e-13)
        np.testing.assert_allclose(dl.sum(1), 0.0, atol=1e-13)  # softmax is shift invariant


def test_route_backward_finite_differences(rng):
    z = rng.standard_normal((4, 6)) * 3
    idx, gate, _ = O.route(z, 2, True)
    dgate = rng.standard_normal(gate.shape)
    dl = O.route_backward(z, idx, gate, dgate, True)
    h = 1e-6
    for t in range(4):
        for e in range(6):
            zp, zm = z.copy(), z.copy()
            zp[t, e] += h
            zm[t, e] -= h
            ip, gp, _ = O.route(zp, 2, True)
            im, gm, _ = O.route(zm, 2, True)
            assert (ip == idx).all() and (im == idx).all()
            fd = ((gp - gm) * dgate).sum() / (2 * h)
            assert abs(fd - dl[t, e]) < 1e-7 * max(1, abs(fd))


def _dispatch_brute(idx, counts, first_slot):
    cls = [int(c) for c in np.asarray(idx).ravel()]
    A, E = len(cls), len(counts)
    rows = sorted(range(A), key=lambda a: (cls[a], a))
    row_of = [0] * A
    for r, a in enumerate(rows):
        row_of[a] = r
    offs = []
    base = 0
    for e in range(E):
        c = cls.count(e)
        for i in range(int(counts[e])):
            offs.append(base + (i * c) // int(counts[e]))
        base += c
    return row_of, rows, offs + [A]


def test_dispatch_matches_brute_force_and_properties(rng):
    for T, E, k, S in [(1, 1, 1, 1), (7, 3, 2, 5), (300, 8, 2, 16), (500, 64, 6, 128), (64, 8, 2, 16)]:
        z = rng.standard_normal((T, E)).astype(np.float32)
        z[:, 0] += 1.5
        if T == 64:
            z[:, 2:] -= 50        # classes 2.. get no token at all
        idx, _, hist = O.route(z, k)
        counts, placement, first = O.place(hist, S)
        row_of, assign_of, offs = O.dispatch(idx, counts, first)
        b_row, b_assign, b_offs = _dispatch_brute(idx, counts, first)
        assert row_of.tolist() == b_row and assign_of.tolist() == b_assign
        assert offs.tolist() == b_offs
        A = T * k
        assert sorted(row_of.tolist()) == list(range(A))                 # bijection
        assert (assign_of[row_of] == np.arange(A)).all()
        cls_rows = idx.ravel()[assign_of]
        assert (np.diff(cls_rows) >= 0).all()                            # grouped by class
        for e in range(E):
            ids = assign_of[cls_rows == e]
            assert (np.diff(ids) > 0).all()                              # stable inside a class
        assert offs[0] == 0 and offs[-1] == A and (np.diff(offs) >= 0).all()
        sizes = np.diff(offs)
        for e in range(E):
            s = sizes[first[e]:first[e + 1]]
            assert s.sum() == hist[e] and s.max() - s.min() <= 1         # near-equal split
            # every row of a slot belongs to the slot's class
            for q in range(first[e], first[e + 1]):
                assert (cls_rows[offs[q]:offs[q + 1]] == placement[q]).all()
