"""Pins for the oracle's layer forward/backward (Sec. 2.1) and Adam-to-replicas
(Sec. 3.2 steps 4-8; Sec. 3.3 weight-phase volume)."""
import numpy as np
import torch

from oracle import symi_oracle as O


def _problem(rng, T=24, E=4, k=2, d=6, f=5, scale=0.5):
    X = rng.standard_normal((T, d))
    W1 = rng.standard_normal((E, 2 * f, d)) * scale
    W2 = rng.standard_normal((E, d, f)) * scale
    z = rng.standard_normal((T, E)) * 2
    idx, gate, hist = O.route(z, k)
    dY = rng.standard_normal((T, d))
    return X, W1, W2, z, idx, gate, hist, dY


def _torch_layer(X, W1, W2, z, idx, renorm=True):
    """The layer written with torch ops only (autograd then derives every gradient)."""
    f = W2.shape[2]
    p = torch.softmax(z, dim=1)
    g = torch.gather(p, 1, idx)
    if renorm:
        g = g / g.sum(1, keepdim=True)
    Y = torch.zeros_like(X)
    for t in range(X.shape[0]):
        for j in range(idx.shape[1]):
            e = int(idx[t, j])
            u = W1[e, :f] @ X[t]
            v = W1[e, f:] @ X[t]
            Y[t] = Y[t] + g[t, j] * (W2[e] @ (torch.nn.functional.silu(u) * v))
    return Y


def test_forward_batched_equals_per_token_loop_and_torch(rng):
    X, W1, W2, z, idx, gate, hist, dY = _problem(rng)
    Y = O.moe_forward(X, idx, gate, W1, W2)
    np.testing.assert_allclose(Y, O.moe_forward_pertoken(X, idx, gate, W1, W2), rtol=1e-12, atol=1e-14)
    Yt = _torch_layer(torch.tensor(X), torch.tensor(W1), torch.tensor(W2), torch.tensor(z),
                      torch.tensor(idx, dtype=torch.int64))
    np.testing.assert_allclose(Y, Yt.numpy(), rtol=1e-11, atol=1e-13)


def test_single_expert_reduces_to_dense_swiglu_mlp(rng):
    T, d, f = 10, 7, 9
    X = rng.standard_normal((T, d))
    W1 = rng.standard_normal((1, 2 * f, d))
    W2 = rng.standard_normal((1, d, f))
    idx, gate, _ = O.route(np.zeros((T, 1)), 1)
    assert (gate == 1).all()
    Y = O.moe_forward(X, idx, gate, W1, W2)
    Xt = torch.tensor(X)
    ref = (torch.nn.functional.silu(Xt @ torch.tensor(W1[0, :f]).T) * (Xt @ torch.tensor(W1[0, f:]).T)) \
        @ torch.tensor(W2[0]).T
    np.testing.assert_allclose(Y, ref.numpy(), rtol=1e-12, atol=1e-13)


def test_backward_against_autograd(rng):
    X, W1, W2, z, idx, gate, hist, dY = _problem(rng)
    dX, dW1, dW2, dgate = O.moe_backward(X, idx, gate, W1, W2, dY)
    dlogits = O.route_backward(z, idx, gate, dgate)
    Xt, W1t, W2t, zt = (torch.tensor(a, requires_grad=True) for a in (X, W1, W2, z))
    Y = _torch_layer(Xt, W1t, W2t, zt, torch.tensor(idx, dtype=torch.int64))
    (Y * torch.tensor(dY)).sum().backward()
    np.testing.assert_allclose(dX, Xt.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dW1, W1t.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dW2, W2t.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dlogits, zt.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dlogits.sum(1), 0, atol=1e-12)


def test_backward_finite_differences(rng):
    X, W1, W2, z, idx, gate, hist, dY = _problem(rng, T=6, E=3, k=2, d=4, f=3)
    dX, dW1, dW2, dgate = O.moe_backward(X, idx, gate, W1, W2, dY)

    def loss(X_, W1_, W2_, gate_):
        return (O.moe_forward(X_, idx, gate_, W1_, W2_) * dY).sum()

    h = 1e-6
    for arr, grad, which in [(X, dX, 0), (W1, dW1, 1), (W2, dW2, 2), (gate, dgate, 3)]:
        it = np.nditer(arr, flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            args = [X, W1, W2, gate]
            ap, am = arr.copy(), arr.copy()
            ap[i] += h
            am[i] -= h
            args[which] = ap
            lp = loss(*args)
            args[which] = am
            lm = loss(*args)
            fd = (lp - lm) / (2 * h)
            assert abs(fd - grad[i]) <= 1e-6 * max(1.0, abs(fd)), (which, i, fd, grad[i])


def test_class_without_tokens_has_zero_gradient(rng):
    X, W1, W2, z, idx, gate, hist, dY = _problem(rng, E=6)
    z[:, 4] = -100.0
    idx, gate, hist = O.route(z, 2)
    assert hist[4] == 0
    _, dW1, dW2, _ = O.moe_backward(X, idx, gate, W1, W2, dY)
    assert not dW1[4].any() and not dW2[4].any()


def test_hidden_units_are_independent_in_the_weight_gradient(rng):
    """dW restricted to a range of hidden units equals the gradient of the FFN that
    keeps only those units (used for sampled full-size parity checks)."""
    X, W1, W2, z, idx, gate, hist, dY = _problem(rng, f=8)
    f = 8
    _, dW1, dW2, _ = O.moe_backward(X, idx, gate, W1, W2, dY)
    sl = slice(2, 5)
    W1s = np.concatenate([W1[:, :f][:, sl], W1[:, f:][:, sl]], axis=1)
    _, dW1s, dW2s, _ = O.moe_backward(X, idx, gate, W1s, W2[:, :, sl], dY)
    np.testing.assert_allclose(dW1s[:, :3], dW1[:, :f][:, sl], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(dW1s[:, 3:], dW1[:, f:][:, sl], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(dW2s, dW2[:, :, sl], rtol=1e-12, atol=1e-14)


HP = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0, grad_scale=1.0, step=1)


def test_adam_against_torch_optim(rng):
    for wd in (0.0, 0.05):
        w0 = rng.standard_normal(50)
        p = torch.tensor(w0, requires_grad=True)
        opt = torch.optim.AdamW([p], lr=1e-2, betas=(0.9, 0.999), eps=1e-8, weight_decay=wd)
        w, m, v = w0.copy(), np.zeros(50), np.zeros(50)
        for step in range(1, 6):
            g = rng.standard_normal(50)
            p.grad = torch.tensor(g)
            opt.step()
            w, m, v = O.adam_step(w, m, v, g, 1e-2, 0.9, 0.999, 1e-8, wd, 1.0, step)
            np.testing.assert_allclose(w, p.detach().numpy(), rtol=1e-12, atol=1e-14)


def test_adam_first_step_closed_form(rng):
    g = rng.standard_normal(20)
    w = rng.standard_normal(20)
    w2, m2, v2 = O.adam_step(w, 0 * w, 0 * w, g, 1e-3, 0.9, 0.999, 1e-8, 0.0, 1.0, 1)
    np.testing.assert_allclose(w2 - w, -1e-3 * g / (np.abs(g) + 1e-8), rtol=1e-9)
    # grad_scale multiplies the gradient before anything else
    w3, m3, _ = O.adam_step(w, 0 * w, 0 * w, g, 1e-3, 0.9, 0.999, 1e-8, 0.0, 0.25, 1)
    np.testing.assert_allclose(m3, 0.25 * m2, rtol=1e-12)


def test_round_to_bf16_matches_torch_cast(rng):
    x = np.concatenate([rng.standard_normal(5000).astype(np.float32) * 3,
                        np.array([1.00390625, 1.01171875, 0.0, -0.0, 3.3895314e38], np.float32)])
    ref = torch.tensor(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert (O.round_to_bf16(x).view(np.uint32) == ref.view(np.uint32)).all()


def test_adam_to_replicas_scatter(rng):
    E, d, f, N, S = 3, 4, 6, 4, 7
    P_e = 3 * d * f
    dW1 = rng.standard_normal((E, 2 * f, d))
    dW2 = rng.standard_normal((E, d, f))
    full_w = rng.standard_normal((E, P_e))
    placement_next = np.array([0, 0, 0, 1, 2, 2, 2], np.int32)
    for bf16 in (False, True):
        W1s = np.full((S, 2 * f, d), 7.0, np.float32)
        W2s = np.full((S, d, f), 7.0, np.float32)
        for n in range(N):
            lo, hi = O.shard_range(P_e, N, n)
            assert (lo, hi) == (n * P_e // N, (n + 1) * P_e // N)
            w, m, v = full_w[:, lo:hi], np.zeros((E, hi - lo)), np.zeros((E, hi - lo))
            before1, before2 = W1s.copy(), W2s.copy()
            w2, m2, v2 = O.adam_to_replicas(dW1, dW2, w, m, v, placement_next, N, n, HP, bf16, W1s, W2s)
            # only partition n's flat range of every slot changed; same count for every slot
            ch = np.concatenate([(W1s != before1).reshape(S, -1), (W2s != before2).reshape(S, -1)], 1)
            assert not ch[:, :lo].any() and not ch[:, hi:].any() and ch[:, lo:hi].all()
            g = np.concatenate([dW1.reshape(E, -1), dW2.reshape(E, -1)], 1)[:, lo:hi]
            np.testing.assert_allclose(w2 - w, -1e-3 * g / (np.abs(g) + 1e-8), rtol=1e-9)
        slots = np.concatenate([W1s.reshape(S, -1), W2s.reshape(S, -1)], 1)
        # after all N partitions every slot holds its class's fresh weights
        gall = np.concatenate([dW1.reshape(E, -1), dW2.reshape(E, -1)], 1)
        fresh = full_w - 1e-3 * gall / (np.abs(gall) + 1e-8)
        want = fresh[placement_next].astype(np.float32)
        if bf16:
            want = torch.tensor(want).to(torch.bfloat16).to(torch.float32).numpy()
            assert (np.abs(slots - want) <= 2.0 ** -8 * np.abs(want)).all()   # at most 1 bf16 ulp
            assert (slots != want).mean() < 0.01
        else:
            np.testing.assert_allclose(slots, want, rtol=1e-6)
