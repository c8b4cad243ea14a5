"""Pins for the oracle's router (a linear layer, Sec. 2.1): torch's linear + autograd, a
finite difference, and the derivative of the whole layer X -> Y taken by torch autograd,
which fixes how the router's dX joins the experts' dX."""
import numpy as np
import torch

from oracle import symi_oracle as O


def _case(seed, T=12, E=5, d=7, k=2, f=3):
    rng = np.random.default_rng(seed)
    return dict(X=rng.standard_normal((T, d)), Wr=rng.standard_normal((E, d)) * 0.5, b=rng.standard_normal(E),
                W1=rng.standard_normal((E, 2 * f, d)) * 0.4, W2=rng.standard_normal((E, d, f)) * 0.4,
                dY=rng.standard_normal((T, d)), k=k)


def test_router_matches_torch_linear_and_autograd():
    c = _case(0)
    X = torch.tensor(c["X"], requires_grad=True); Wr = torch.tensor(c["Wr"], requires_grad=True)
    b = torch.tensor(c["b"], requires_grad=True)
    z = torch.nn.functional.linear(X, Wr, b)
    np.testing.assert_allclose(O.router_forward(c["X"], c["Wr"], c["b"]), z.detach().numpy(), rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(O.router_forward(c["X"], c["Wr"]), (z - b).detach().numpy(), rtol=1e-13, atol=1e-13)
    dl = np.random.default_rng(1).standard_normal(z.shape)
    (z * torch.tensor(dl)).sum().backward()
    dWr, db, dX = O.router_backward(c["X"], c["Wr"], dl)
    np.testing.assert_allclose(dWr, Wr.grad.numpy(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(db, b.grad.numpy(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(dX, X.grad.numpy(), rtol=1e-12, atol=1e-12)


def test_router_finite_difference():
    c = _case(2)
    dl = np.random.default_rng(3).standard_normal((c["X"].shape[0], c["Wr"].shape[0]))
    loss = lambda Wr: (O.router_forward(c["X"], Wr, c["b"]) * dl).sum()
    dWr, _, _ = O.router_backward(c["X"], c["Wr"], dl)
    for e, j in [(0, 0), (3, 5), (4, 6)]:
        Wp, Wm = c["Wr"].copy(), c["Wr"].copy()
        Wp[e, j] += 1e-6; Wm[e, j] -= 1e-6
        assert abs((loss(Wp) - loss(Wm)) / 2e-6 - dWr[e, j]) < 1e-6


def test_whole_layer_gradient_from_X_through_router_and_experts():
    c = _case(5)
    k = c["k"]
    z = O.router_forward(c["X"], c["Wr"], c["b"])
    idx, gate, _ = O.route(z, k, True)
    Y = O.moe_forward(c["X"], idx, gate, c["W1"], c["W2"])
    dX_e, _, _, dgate = O.moe_backward(c["X"], idx, gate, c["W1"], c["W2"], c["dY"])
    dlogits = O.route_backward(z, idx, gate, dgate, True)
    dWr, db, dX_r = O.router_backward(c["X"], c["Wr"], dlogits)
    # the same function in torch (choices held fixed), differentiated automatically
    t = {n: torch.tensor(c[n], requires_grad=n in ("X", "Wr", "b")) for n in ("X", "Wr", "b", "W1", "W2", "dY")}
    zt = t["X"] @ t["Wr"].T + t["b"]
    p = torch.softmax(zt, dim=1)
    ii = torch.tensor(idx.astype(np.int64))
    g = torch.gather(p, 1, ii)
    g = g / g.sum(dim=1, keepdim=True)
    f = c["W2"].shape[2]
    Yt = torch.zeros_like(t["X"])
    for tok in range(c["X"].shape[0]):
        for j in range(k):
            e = int(idx[tok, j])
            u = t["W1"][e, :f] @ t["X"][tok]; v = t["W1"][e, f:] @ t["X"][tok]
            Yt[tok] = Yt[tok] + g[tok, j] * (t["W2"][e] @ (torch.nn.functional.silu(u) * v))
    np.testing.assert_allclose(Y, Yt.detach().numpy(), rtol=1e-11, atol=1e-11)
    (Yt * t["dY"]).sum().backward()
    np.testing.assert_allclose(dX_e + dX_r, t["X"].grad.numpy(), rtol=1e-9, atol=1e-10)
    np.testing.assert_allclose(dWr, t["Wr"].grad.numpy(), rtol=1e-9, atol=1e-10)
    np.testing.assert_allclose(db, t["b"].grad.numpy(), rtol=1e-9, atol=1e-10)
