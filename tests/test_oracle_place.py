"""Pins for the oracle's placement (Algorithm 1, App. A.3; Sec. 3.4)."""
import os
import random
from fractions import Fraction

import numpy as np
import pytest

from oracle import symi_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "placement_cases.txt")


def _golden_cases():
    out = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        s, pop, exp = line.split("|")
        out.append((int(s), [int(x) for x in pop.split()], [int(x) for x in exp.split()]))
    return out


@pytest.mark.parametrize("S_tot,pop,expected", _golden_cases())
def test_golden_cases(S_tot, pop, expected):
    counts, placement, first = O.place(pop, S_tot)
    assert counts.tolist() == expected
    assert placement.tolist() == [e for e, c in enumerate(expected) for _ in range(c)]
    assert first.tolist() == [0] + list(np.cumsum(expected))


def _compositions(S, E):
    if E == 1:
        yield (S,)
        return
    for a in range(1, S - E + 2):
        for rest in _compositions(S - a, E - 1):
            yield (a,) + rest


def test_invariants_random():
    rnd = random.Random(7)
    for _ in range(3000):
        E = rnd.randint(1, 40)
        S = rnd.randint(E, 4 * E + 5)
        pop = [rnd.choice([0, 0, 1, 3, rnd.randint(0, 5000)]) for _ in range(E)]
        counts, placement, first = O.place(pop, S)
        assert counts.min() >= 1                      # every class reachable
        assert counts.sum() == S                      # slot budget used exactly
        assert len(placement) == S
        assert np.all(np.diff(placement) >= 0)        # same-class slots contiguous
        assert np.bincount(placement, minlength=E).tolist() == counts.tolist()
        assert first[0] == 0 and first[-1] == S
        assert np.all(np.diff(first) == counts)


def test_brute_force_optimal_on_tiny_inputs():
    """Among all count vectors >= 1 summing to S_tot the result minimises both the
    largest over-allocation max_i(counts_i - goal_i) and the L1 distance to the goal."""
    rnd = random.Random(11)
    for _ in range(1500):
        E = rnd.randint(1, 4)
        S = rnd.randint(E, 12)
        pop = [rnd.randint(0, 20) for _ in range(E)]
        if sum(pop) == 0:
            continue
        counts = O.place(pop, S)[0].tolist()
        goal = [Fraction(p * S, sum(pop)) for p in pop]
        best_over = min(max(c - g for c, g in zip(cc, goal)) for cc in _compositions(S, E))
        best_l1 = min(sum(abs(c - g) for c, g in zip(cc, goal)) for cc in _compositions(S, E))
        assert max(c - g for c, g in zip(counts, goal)) == best_over, (pop, S, counts)
        assert sum(abs(c - g) for c, g in zip(counts, goal)) == best_l1, (pop, S, counts)


def _hamilton(pop, S):
    """Largest-remainder apportionment, ties to the lowest index."""
    P = sum(pop)
    goal = [Fraction(p * S, P) for p in pop]
    fl = [int(g) for g in goal]
    order = sorted(range(len(pop)), key=lambda i: (-(goal[i] - fl[i]), i))
    for i in order[: S - sum(fl)]:
        fl[i] += 1
    return fl


def test_reduces_to_hamilton_when_no_class_is_lifted():
    rnd = random.Random(3)
    n = 0
    for _ in range(4000):
        E = rnd.randint(1, 16)
        S = rnd.randint(E, 6 * E)
        pop = [rnd.randint(1, 300) for _ in range(E)]
        if min(p * S for p in pop) < sum(pop):      # some goal < 1: min-1 rule active
            continue
        n += 1
        assert O.place(pop, S)[0].tolist() == _hamilton(pop, S)
    assert n > 300


def test_uniform_popularity_is_the_static_baseline():
    # eq. (1): r = sN/E when popularity is uniform and E divides the slot budget
    for E, S in [(8, 16), (16, 64), (64, 128), (128, 256)]:
        assert O.place([17] * E, S)[0].tolist() == [S // E] * E
    # no popularity yet (first iteration) is read as uniform
    assert O.place([0] * 8, 16)[0].tolist() == [2] * 8
    c = O.place([0] * 64, 96)[0].tolist()
    assert c == [2] * 32 + [1] * 32


def test_exact_tie_between_two_diffs_goes_to_the_first_class():
    """(10,3,10,5) at 16 slots: goals 5.71, 1.71, 5.71, 2.86 floor to 5,1,5,2 (13 slots); the
    three missing replicas go to the most under-served classes: class 3 (diff -0.86), then
    classes 0, 1 and 2 tie at -0.71 exactly and the first two of them win."""
    assert O.place([10, 3, 10, 5], 16)[0].tolist() == [6, 2, 5, 3]


def test_rejects_too_few_slots():
    with pytest.raises(ValueError):
        O.place([1, 2, 3], 2)
