"""Pins for the oracle's replica gradient path (Sec. 4.1): the per-slot gradients add up to
the class gradient of the plain definition, whatever the placement; after the all-reduce
every replica holds that sum (times the scale)."""
import numpy as np

from oracle import symi_oracle as O


def _case(seed, E=4, S=9, T=40, k=2, d=6, f=5):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((T, d)); dY = rng.standard_normal((T, d))
    W1 = rng.standard_normal((E, 2 * f, d)) * 0.3; W2 = rng.standard_normal((E, d, f)) * 0.3
    logits = rng.standard_normal((T, E)) + np.array([2.0, 0.5, 0, 0])[:E]
    idx, gate, hist = O.route(logits, k, True)
    counts, placement, first = O.place(rng.multinomial(T * k, np.full(E, 1 / E)), S)
    roa, aor, off = O.dispatch(idx, counts, first)
    return X, dY, W1, W2, idx, gate, counts, placement, first, roa, off


def test_slot_gradients_sum_to_the_class_gradient():
    for seed in range(4):
        X, dY, W1, W2, idx, gate, counts, placement, first, roa, off = _case(seed)
        g1, g2 = O.slot_gradients(X, idx, gate, W1, W2, dY, roa, off)
        _, dW1, dW2, _ = O.moe_backward(X, idx, gate, W1, W2, dY)
        for e in range(len(counts)):
            np.testing.assert_allclose(g1[first[e]:first[e + 1]].sum(0), dW1[e], rtol=1e-12, atol=1e-12)
            np.testing.assert_allclose(g2[first[e]:first[e + 1]].sum(0), dW2[e], rtol=1e-12, atol=1e-12)
        # an empty slot has no gradient
        for q in np.nonzero(np.diff(off) == 0)[0]:
            assert not g1[q].any() and not g2[q].any()


def test_replica_allreduce_leaves_the_scaled_class_sum_in_every_slot():
    X, dY, W1, W2, idx, gate, counts, placement, first, roa, off = _case(11)
    g1, _ = O.slot_gradients(X, idx, gate, W1, W2, dY, roa, off)
    _, dW1, _, _ = O.moe_backward(X, idx, gate, W1, W2, dY)
    for scale in (1.0, 0.25):
        r = O.replica_allreduce(g1, first, scale)
        for q, e in enumerate(placement):
            np.testing.assert_allclose(r[q], scale * dW1[e], rtol=1e-12, atol=1e-12)
    # brute force on a hand-made case: class 0 in slots 0-2, class 1 in slot 3
    g = np.arange(4 * 2, dtype=float).reshape(4, 2)
    r = O.replica_allreduce(g, np.array([0, 3, 4]), 0.5)
    assert (r == np.array([[3.0, 4.5], [3.0, 4.5], [3.0, 4.5], [3.0, 3.5]])).all()
