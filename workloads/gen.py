"""Seeded tensor generators (torch RNG on the requested device).

Every tensor is keyed by (config seed, tensor id, iteration).  A tensor drawn on
`cuda` differs from the same key drawn on `cpu` (different RNG engines); a test
always draws ONCE and hands the same values to both sides (`.cpu()` copies for the
oracle).  bf16 configs round the drawn fp32 values to bf16 here, so that oracle and
kernels start from identical, exactly representable inputs.
"""
import torch

from .configs import Config

_TENSOR_IDS = {"tokens": 1, "router_w": 2, "noise": 3, "w1": 4, "w2": 5, "dy": 6,
               "perm": 7, "walk": 8, "router_wr": 9}


def _gen(cfg: Config, what: str, it: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(1_000_003 * cfg.seed + 10_007 * _TENSOR_IDS[what] + it + 12345)
    return g


def _act_dtype(cfg: Config):
    return torch.float32 if cfg.dtype == "f32" else torch.bfloat16


def make_tokens(cfg: Config, it: int = 0, device="cpu") -> torch.Tensor:
    """X [T, d] ~ N(0, 1) in the config's activation dtype."""
    x = torch.randn(cfg.T, cfg.d, generator=_gen(cfg, "tokens", it, device),
                    device=device, dtype=torch.float32)
    return x.to(_act_dtype(cfg))


def make_upstream_grad(cfg: Config, it: int = 0, device="cpu") -> torch.Tensor:
    """dY [T, d] ~ N(0, 1): the gradient arriving from the layer above."""
    g = torch.randn(cfg.T, cfg.d, generator=_gen(cfg, "dy", it, device),
                    device=device, dtype=torch.float32)
    return g.to(_act_dtype(cfg))


def make_class_weights(cfg: Config, device="cpu", std: float = 0.02):
    """Per-class expert weights: W1 [E, 2f, d] (gate rows, then up rows), W2 [E, d, f]."""
    dt = _act_dtype(cfg)
    w1 = torch.empty(cfg.E, 2 * cfg.f, cfg.d, device=device, dtype=dt)
    w2 = torch.empty(cfg.E, cfg.d, cfg.f, device=device, dtype=dt)
    g1 = _gen(cfg, "w1", 0, device)
    g2 = _gen(cfg, "w2", 0, device)
    for e in range(cfg.E):  # per class, to bound the fp32 staging buffer
        w1[e] = (torch.randn(2 * cfg.f, cfg.d, generator=g1, device=device) * std).to(dt)
        w2[e] = (torch.randn(cfg.d, cfg.f, generator=g2, device=device) * std).to(dt)
    return w1, w2


def bias_schedule(cfg: Config, it: int = 0) -> torch.Tensor:
    """Per-class logit bias b[E] (fp32, CPU) of iteration `it`: the popularity process."""
    E = cfg.E
    if cfg.bias == "zipf":
        # rank weight z_r ~ r^-s; bias = 2*log z_r (normalisation is a constant shift)
        rank = torch.arange(1, E + 1, dtype=torch.float64)
        b = (-2.0 * cfg.zipf_s) * torch.log(rank)
        if cfg.reshuffle:
            perm = torch.randperm(E, generator=_gen(cfg, "perm", it, "cpu"))
            b = b[perm]
        return b.to(torch.float32)
    if cfg.bias == "hot0":
        b = torch.zeros(E, dtype=torch.float32)
        b[0] = cfg.hot_bias
        return b
    if cfg.bias == "walk":
        # b^(0) = 0, b^(i+1) = b^(i) + N(0, walk_sigma^2)
        g = _gen(cfg, "walk", 0, "cpu")
        n = max(cfg.iters, it, 1)  # always draw the whole schedule: prefix-stable
        steps = torch.randn(n, E, generator=g, dtype=torch.float64) * cfg.walk_sigma
        b = steps[:it].sum(0) if it > 0 else torch.zeros(E, dtype=torch.float64)
        return b.to(torch.float32)
    raise ValueError(cfg.bias)


def make_logits(cfg: Config, it: int = 0, device="cpu", tokens: torch.Tensor = None):
    """Router logits [T, E] fp32 of iteration `it`.

    c1 style: X @ W_r + b with W_r ~ N(0, 0.02^2) (fp32 matmul, done here as input
    preparation: the hot path starts at the logits).  Others: N(0, sigma^2) noise + b.
    """
    b = bias_schedule(cfg, it).to(device)
    if cfg.router_matmul:
        if tokens is None:
            tokens = make_tokens(cfg, it, device)
        wr = torch.randn(cfg.d, cfg.E, generator=_gen(cfg, "router_w", 0, device),
                         device=device, dtype=torch.float32) * 0.02
        return (tokens.to(torch.float32) @ wr + b).contiguous()
    noise = torch.randn(cfg.T, cfg.E, generator=_gen(cfg, "noise", it, device),
                        device=device, dtype=torch.float32)
    return (noise * cfg.noise_sigma + b).contiguous()


def make_router(cfg: Config, it: int = 0, device="cpu"):
    """Router parameters for the closed layer: Wr [E, d] ~ N(0, 0.02^2) in the config's
    activation dtype (row e scores class e), b [E] fp32 = the popularity bias of iteration
    `it` (so the routed histogram keeps the config's skew)."""
    wr = torch.randn(cfg.E, cfg.d, generator=_gen(cfg, "router_wr", 0, device), device=device,
                     dtype=torch.float32) * 0.02
    dt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    return wr.to(dt).contiguous(), bias_schedule(cfg, it).to(device).to(torch.float32).contiguous()
