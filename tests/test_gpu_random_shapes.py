"""GPU parity on seeded random shapes: every stage of an iteration against the oracle on
configurations nobody picked by hand (class counts that are no power of two, widths that are no
tile multiple, one token, more slots than rows, several rounds of ragged tiles), with the plain
or the *_active gradient pair, two iterations each so that the second placement mimics the
first iteration's popularity."""
import random

import pytest
import torch

import workloads as wl
import harness as Hn
from tests.checks import check_iteration
import tests.test_gpu_next_edges as next_edges

pytestmark = pytest.mark.gpu


def _legal_f(d, f, N):
    while (3 * d * f) % N or (3 * d * f // N) % 8:
        f += 8
    return f


def _small(rng, i):
    dtype = rng.choice(["bf16", "bf16", "f32"])
    E = rng.choice([1, 2, 3, 8, 16, 24, 64, 130])
    k = rng.randint(1, min(E, 8))
    N = rng.choice([1, 2, 3, 4, 8])
    d = 8 * rng.randint(1, 80)
    f = _legal_f(d, 8 * rng.randint(1, 300 if dtype == "bf16" else 40), N)
    S = ((E + rng.randint(0, 3 * E) + N - 1) // N) * N
    T = rng.choice([1, 7, 130, 300, 777, 1500])
    if dtype == "f32":
        T = min(T, 300)
    return wl.scaled(wl.get_config("c2"), dtype=dtype, E=E, k=k, d=d, f=f, T=T, S_tot=S, N=N, iters=1,
                     router_matmul=False, seed=1100 + i)


def _mid(rng, i):
    E = rng.choice([2, 4, 8, 16])
    k = rng.randint(1, min(E, 3))
    N = rng.choice([1, 2, 4])
    d = 8 * rng.randint(33, 260)
    f = _legal_f(d, 8 * rng.randint(65, 700), N)
    S = ((E + rng.randint(0, E) + N - 1) // N) * N
    return wl.scaled(wl.get_config("c2"), E=E, k=k, d=d, f=f, T=rng.randint(1500, 9000), S_tot=S, N=N,
                     iters=1, router_matmul=False, seed=7200 + i)


@pytest.mark.parametrize("kind,seed,count", [("small", 11, 10), ("small", 12, 12), ("mid", 21, 3)])
def test_random_shapes_full_iteration(kind, seed, count):
    rng = random.Random(seed)
    for i in range(count):
        c = (_small if kind == "small" else _mid)(rng, 100 * seed + i)
        st = Hn.State(c, shard=rng.randrange(c.N))
        st.active_grads = rng.random() < 0.5
        print(f"[random {kind} {seed}/{i}] active={st.active_grads} {c}", flush=True)
        X, logits, dY = Hn.draw_inputs(c, 0)
        check_iteration(st, X, logits, dY)
        if kind == "small":
            st.hist_prev.copy_(st.hist)
            check_iteration(st, X, logits, dY, hp_kw=dict(step=2))
        del st
        torch.cuda.empty_cache()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_random_shapes_router_capacity_replica_path(dtype, monkeypatch):
    rng = random.Random(31 if dtype == "bf16" else 32)

    def cases(dt):
        base = wl.scaled(wl.get_config("c1"), dtype=dt)
        out = []
        for i in range(10):
            E = rng.choice([1, 2, 5, 8, 23, 64, 130, 257])
            k = rng.randint(1, min(E, 8))
            N = rng.choice([1, 2, 4])
            d = 8 * rng.randint(1, 60)
            f = _legal_f(d, 8 * rng.randint(1, 40), N)
            S = ((E + rng.randint(0, 2 * E) + N - 1) // N) * N
            out.append(wl.scaled(base, E=E, k=k, d=d, f=f, T=rng.choice([1, 9, 130, 511, 513, 1200]),
                                 S_tot=S, N=N, router_matmul=False, bias="zipf", zipf_s=1.2, seed=5400 + i))
        return out

    monkeypatch.setattr(next_edges, "_cases", cases)
    next_edges.test_router_capacity_and_replica_path_on_edge_shapes(dtype)
