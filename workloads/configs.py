"""The five synthetic workload shapes (notation of the paper's Table 2).

E  expert classes          k  choices per token      d, f  model / FFN width
T  tokens in the batch     S_tot = s*N replica slots N     optimizer partitions
"""
from dataclasses import dataclass, replace


@dataclass(frozen=True)
class Config:
    name: str
    dtype: str          # "f32" | "bf16": weights and activations (Adam state is fp32)
    E: int
    k: int
    d: int
    f: int
    T: int
    S_tot: int
    N: int
    iters: int
    bias: str           # "zipf" | "hot0" | "walk"
    zipf_s: float = 0.0
    reshuffle: bool = False   # new random popularity ranking every iteration
    hot_bias: float = 0.0
    noise_sigma: float = 1.0
    walk_sigma: float = 0.0
    router_matmul: bool = False  # logits = X @ W_r + b instead of noise + b
    seed: int = 0

    @property
    def A(self) -> int:
        return self.T * self.k

    @property
    def P_e(self) -> int:
        return 3 * self.d * self.f


CONFIGS = {
    # fp32, E=8, top-2, d=128, f=256, T=1024, 16 slots, N=4; logits from a router matmul
    "c1": Config("c1", "f32", 8, 2, 128, 256, 1024, 16, 4, 1, "zipf", zipf_s=1.2,
                 router_matmul=True, seed=0),
    # bf16, E=64, top-2, d=1024, f=4096, T=8192, 96 slots, N=8; ranking reshuffled, 10 iters
    "c2": Config("c2", "bf16", 64, 2, 1024, 4096, 8192, 96, 8, 10, "zipf", zipf_s=1.2,
                 reshuffle=True, seed=2),
    # bf16, E=8, top-2, d=4096, f=14336, T=16384, 16 slots, N=8; expert 0 gets ~40 % of assignments
    "c3": Config("c3", "bf16", 8, 2, 4096, 14336, 16384, 16, 8, 1, "hot0", hot_bias=3.0,
                 noise_sigma=1.7, seed=3),
    # bf16, E=64, top-6, d=2048, f=1408, T=32768, 128 slots, N=16; bias random walk, 20 iters
    "c4": Config("c4", "bf16", 64, 6, 2048, 1408, 32768, 128, 16, 20, "walk", walk_sigma=0.3,
                 seed=4),
    # bf16, E=128, top-8, d=4096, f=2048, T=65536, 256 slots, N=32; near-uniform Zipf 0.5
    "c5": Config("c5", "bf16", 128, 8, 4096, 2048, 65536, 256, 32, 1, "zipf", zipf_s=0.5,
                 seed=5),
}


def get_config(name: str) -> Config:
    return CONFIGS[name]


def scaled(cfg: Config, **kw) -> Config:
    """Same recipe at other sizes (parity tests shrink T, d or f; E, k stay)."""
    return replace(cfg, **kw)
