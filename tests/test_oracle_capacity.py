"""Pins for the oracle's capacity rule (Sec. 3.4): slot_capacity, dispatch_capacity.

Independent checks: a literal first-come-first-kept loop, the invariants the rule implies,
reduction to the dropless dispatch, the paper's identity between the per-class and the
per-slot form of the capacity, closed-form survival for uniform and for exactly
proportional placements.
"""
from fractions import Fraction

import numpy as np
import pytest

from oracle import symi_oracle as O


def _first_slot(counts):
    return np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)


def _random_case(rng, E, S, T, k, skew):
    p = rng.dirichlet(np.full(E, skew))
    idx = np.stack([rng.choice(E, size=k, replace=False, p=p) for _ in range(T)]).astype(np.int32)
    hist_prev = rng.multinomial(T * k, rng.dirichlet(np.full(E, skew)))
    counts, _, first = O.place(hist_prev, S)
    return idx, counts, first


def _literal(idx, counts, first_slot, slot_cap):
    """Walk the assignments in order; a class accepts them until it is full."""
    cls = np.asarray(idx).ravel()
    E = len(counts)
    seen = [0] * E
    keep = []
    for a in range(cls.size):
        e = int(cls[a])
        ok = seen[e] < slot_cap * int(counts[e])
        keep.append(ok)
        seen[e] += ok
    kept = [[a for a in range(cls.size) if keep[a] and cls[a] == e] for e in range(E)]
    rows = [a for e in range(E) for a in kept[e]]
    roa = [-1] * cls.size
    for r, a in enumerate(rows):
        roa[a] = r
    return np.array(roa), np.array(rows), np.array(keep), [len(x) for x in kept]


@pytest.mark.parametrize("seed", range(12))
def test_matches_literal_first_come_first_kept(seed):
    rng = np.random.default_rng(seed)
    E = int(rng.integers(2, 9)); k = int(rng.integers(1, min(E, 3) + 1))
    S = int(rng.integers(E, 3 * E + 1)); T = int(rng.integers(1, 120))
    idx, counts, first = _random_case(rng, E, S, T, k, 0.4)
    for cf in (0.3, 1.0, 1.7):
        cap = O.slot_capacity(cf, T * k, S)
        roa, aor, off, keep = O.dispatch_capacity(idx, counts, first, cap)
        l_roa, l_rows, l_keep, l_kept = _literal(idx, counts, first, cap)
        assert (roa == l_roa).all() and (aor == l_rows).all() and (keep == l_keep).all()
        # slot boundaries: class e's kept rows in r_e near-equal contiguous blocks, none above cap
        sizes = np.diff(off)
        assert off[0] == 0 and off[-1] == sum(l_kept) and (sizes >= 0).all() and sizes.max(initial=0) <= cap
        for e in range(E):
            sz = sizes[first[e]:first[e + 1]]
            assert sz.sum() == l_kept[e] and sz.max() - sz.min() <= 1


def test_invariants_on_a_larger_case():
    rng = np.random.default_rng(7)
    E, S, T, k = 64, 96, 4096, 2
    idx, counts, first = _random_case(rng, E, S, T, k, 0.2)
    cap = O.slot_capacity(1.0, T * k, S)
    roa, aor, off, keep = O.dispatch_capacity(idx, counts, first, cap)
    cls = idx.ravel()
    c = np.bincount(cls, minlength=E)
    kept = np.bincount(cls[keep], minlength=E)
    assert (kept == np.minimum(c, cap * counts)).all()
    assert (roa[keep] >= 0).all() and (roa[~keep] == -1).all()
    assert (roa[aor] == np.arange(aor.size)).all()                 # inverse on the kept rows
    assert (np.diff(cls[aor]) >= 0).all()                          # classes ascend along the rows
    for e in range(E):                                             # assignment ids ascend in a class
        a = aor[cls[aor] == e]
        assert (np.diff(a) > 0).all()
        dropped = np.nonzero((cls == e) & ~keep)[0]
        if dropped.size and a.size:
            assert dropped.min() > a.max()                         # the kept ones are the first ones
    assert 0 < keep.mean() < 1


def test_unbounded_capacity_is_the_dropless_dispatch():
    rng = np.random.default_rng(3)
    idx, counts, first = _random_case(rng, 16, 40, 700, 2, 0.3)
    roa0, aor0, off0 = O.dispatch(idx, counts, first)
    roa, aor, off, keep = O.dispatch_capacity(idx, counts, first, 10 ** 6)
    assert keep.all() and (roa == roa0).all() and (aor == aor0).all() and (off == off0).all()


def test_slot_capacity_values_and_per_class_identity():
    # config c2: 16384 assignments over 96 slots
    assert O.slot_capacity(1.0, 16384, 96) == 171          # ceil(170.67)
    assert O.slot_capacity(1.5, 16384, 96) == 256          # exact
    assert O.slot_capacity(2.0, 16384, 96) == 342
    assert O.slot_capacity(1.0, 1024, 128) == 8
    assert O.slot_capacity(1e-9, 16, 16) == 1              # never below one row
    # Sec. 3.4, identity (1): capacity_factor * tokens / E == slot_capacity * r with r = s*N/E
    for cf, A, E, S in [(Fraction(1), 8192, 64, 128), (Fraction(5, 4), 4096, 8, 16), (Fraction(2), 300, 10, 40)]:
        r = Fraction(S, E)
        assert cf * A / E == (cf * A / S) * r


def test_survival_closed_forms():
    E, S, k = 8, 16, 1
    # popularity exactly proportional to the replicas: nothing is dropped at capacity_factor 1
    counts = np.array([5, 3, 2, 2, 1, 1, 1, 1], dtype=np.int32)
    per_slot = 12
    cls = np.repeat(np.arange(E), counts * per_slot)
    rng = np.random.default_rng(0)
    rng.shuffle(cls)
    idx = cls.reshape(-1, k).astype(np.int32)
    A = cls.size
    cap = O.slot_capacity(1.0, A, S)
    assert cap == per_slot
    _, aor, off, keep = O.dispatch_capacity(idx, counts, _first_slot(counts), cap)
    assert keep.all() and (np.diff(off) == per_slot).all()
    # the same tokens under the static uniform placement (r = S/E = 2 each):
    # survival = sum_e min(c_e, capacity_factor * A / E) / A
    uni = np.full(E, S // E, dtype=np.int32)
    _, _, _, keep_u = O.dispatch_capacity(idx, uni, _first_slot(uni), cap)
    c = counts * per_slot
    assert keep_u.sum() == np.minimum(c, A // E).sum()
    assert keep_u.mean() == pytest.approx(np.minimum(c, A / E).sum() / A)
