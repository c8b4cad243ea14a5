"""CPU-only checks of the C ABI: the library loads, exports every declared symbol, and
its host-side entry points (validation, workspace size, the host scheduler) behave."""
import os
import random
import re

import numpy as np
import pytest
import torch

import paper_2504_19925_amd as symi
from oracle import symi_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "symi.h")).read()
    declared = sorted(set(re.findall(r"\b(symi_[a-z_0-9]+)\s*\(", header)))
    assert declared == sorted(symi.EXPORTS)
    L = symi.lib()
    for name in declared:
        assert hasattr(L, name), name


def _cfg(**kw):
    base = dict(T=64, E=8, k=2, d=128, f=256, S_tot=16, N=4, shard=0, dtype="f32", renorm=1)
    base.update(kw)
    return symi.SymiCfg.make(**base)


def test_validate_accepts_the_five_configs_and_rejects_bad_shapes():
    from workloads import CONFIGS
    for c in CONFIGS.values():
        cfg = symi.SymiCfg.make(c.T, c.E, c.k, c.d, c.f, c.S_tot, c.N, 0, c.dtype, 1)
        assert symi.symi_validate(cfg) == 0
        assert symi.symi_workspace_bytes(cfg) > 0
    for bad in (dict(S_tot=7), dict(k=9), dict(k=0), dict(shard=4), dict(N=0), dict(d=100),
                dict(f=12), dict(N=7), dict(E=0), dict(T=-1)):
        cfg = _cfg(**bad)
        assert symi.symi_validate(cfg) == -1, bad
        assert symi.symi_last_error() != ""
        assert symi.symi_workspace_bytes(cfg) == 0


def test_place_host_matches_oracle():
    rnd = random.Random(42)
    cases = [([5, 5, 4, 2], 16), ([1024, 1024, 0, 0, 0, 0, 0, 0], 16), ([0] * 64, 96),
             ([10, 3, 10, 5], 16), ([1000000] + [0] * 63, 64)]
    for _ in range(1500):
        E = rnd.randint(1, 130)
        S = rnd.randint(E, 3 * E + 2)
        cases.append(([rnd.choice([0, 1, 2, rnd.randint(0, 60000)]) for _ in range(E)], S))
    for pop, S in cases:
        E = len(pop)
        cfg = symi.SymiCfg.make(64, E, 1, 128, 256, S, 1, 0, "f32", 1)
        counts = torch.zeros(E, dtype=torch.int32)
        placement = torch.zeros(S, dtype=torch.int32)
        first = torch.zeros(E + 1, dtype=torch.int32)
        symi.symi_place_host(cfg, torch.tensor(pop, dtype=torch.int32), counts, placement, first)
        oc, op, of = O.place(pop, S)
        assert counts.tolist() == oc.tolist(), (pop, S)
        assert placement.tolist() == op.tolist()
        assert first.tolist() == of.tolist()


def test_binding_refuses_cpu_tensors_for_device_calls():
    ctx = symi.SymiCtx(None, _cfg(), 0)     # never reaches the library: the tensors are refused first
    z = torch.zeros(64, 8)
    with pytest.raises(symi.SymiError):
        symi.symi_route(ctx, z, torch.zeros(64, 2, dtype=torch.int32), torch.zeros(64, 2),
                        torch.zeros(8, dtype=torch.int32))


def test_context_create_and_destroy():
    """symi_create validates on the host before it touches a device; without a usable device it
    fails with SYMI_EHIP and a message; device calls refuse a NULL context; destroying NULL is
    allowed.  With a GPU: contexts are created and destroyed repeatedly, with every flag."""
    import ctypes
    L = symi.lib()
    out = ctypes.c_void_p()
    assert L.symi_create(None, 0, ctypes.byref(out)) == -1 and not out.value
    assert L.symi_create(ctypes.byref(_cfg()), 0, None) == -1
    assert L.symi_create(ctypes.byref(_cfg(S_tot=7)), 0, ctypes.byref(out)) == -1 and not out.value
    assert L.symi_create(ctypes.byref(_cfg()), 8, ctypes.byref(out)) == -1      # unknown flag bit
    assert "flag" in symi.symi_last_error()
    assert L.symi_destroy(None) == 0
    assert L.symi_route(None, None, None, None, None, None) == -1
    assert "ctx" in symi.symi_last_error()
    assert L.symi_timing_reset(None) == -1
    if not torch.cuda.is_available():
        with pytest.raises(symi.SymiError, match="device"):
            symi.symi_create(_cfg())
        assert L.symi_create(ctypes.byref(_cfg()), 0, ctypes.byref(out)) == -3 and not out.value
        return
    for flags in (0, symi.CTX_NO_OVERLAP, symi.CTX_NO_SLICING, symi.CTX_TIMING,
                  symi.CTX_NO_OVERLAP | symi.CTX_NO_SLICING | symi.CTX_TIMING) * 3:
        ctx = symi.symi_create(_cfg(dtype="bf16"), flags)
        assert ctx.ptr and ctx.T == 64 and ctx.flags == flags
        symi.symi_destroy(ctx)
        assert ctx.ptr is None
        symi.symi_destroy(ctx)               # a second destroy of the handle is a no-op


def test_launch_limits_are_rejected_as_unsupported():
    """Shapes whose grids or 32-bit offsets the kernels cannot address are refused up front."""
    ok = dict(T=1 << 20, E=8, k=8, d=64, f=64, S_tot=16, N=1, dtype="bf16")
    assert symi.symi_validate(_cfg(**ok)) == 0
    for bad in (dict(ok, T=1 << 22, k=4),                 # 65536 + 16 + 256 m-tiles
                dict(ok, dtype="f32"),                    # fp32 tiles are a quarter the rows
                dict(ok, T=(1 << 23) + 1024, k=1, E=1, S_tot=1),   # T / 128 > 65535
                dict(ok, T=64, d=1 << 16, f=1 << 14),     # 2*f*d = 2^31
                dict(ok, T=64, d=8, f=(1 << 27) - 8),     # 2*f*d = 2^31 - 128: no room for the offset bias
                dict(ok, T=64, d=1 << 23, f=8),           # 256 rows of d elements pass 2^32 bytes
                dict(ok, T=64, d=8, f=1 << 22)):          # ... of 2f elements
        assert symi.symi_validate(_cfg(**bad)) == -2, bad
        assert symi.symi_workspace_bytes(_cfg(**bad)) == 0


def test_slot_capacity_host_function_matches_oracle():
    """symi_slot_capacity is a host computation: Sec. 3.4's slot_capacity, rounded up."""
    rng = random.Random(5)
    for _ in range(500):
        E = rng.randint(1, 64)
        S = rng.randint(E, 4 * E)
        k = rng.randint(1, min(E, 8))
        T = rng.randint(0, 5000)
        cfg = symi.SymiCfg.make(T=T, E=E, k=k, d=64, f=64, S_tot=S, N=1, shard=0, dtype="f32")
        cf = rng.choice([0.25, 0.5, 1.0, 1.25, 1.5, 2.0, 4.0, rng.uniform(0.01, 8.0)])
        assert symi.symi_slot_capacity(cfg, cf) == O.slot_capacity(cf, T * k, S)
    cfg = symi.SymiCfg.make(T=8192, E=64, k=2, d=1024, f=4096, S_tot=96, N=8, shard=0, dtype="bf16")
    assert symi.symi_slot_capacity(cfg, 1.0) == 171 and symi.symi_slot_capacity(cfg, 1.5) == 256
    for bad in (0.0, -1.0, float("nan")):
        with pytest.raises(symi.SymiError):
            symi.symi_slot_capacity(cfg, bad)
