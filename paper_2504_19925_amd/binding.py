"""ctypes binding of libsymi.so: same names as the C ABI, argument marshalling only.

Tensors must live on the GPU (except where the C function takes host pointers), be
contiguous and have the dtype the header states; the current torch stream is passed
through.  There is no fallback: if the library is missing or a call fails, SymiError
is raised.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

EXPORTS = [
    "symi_validate", "symi_create", "symi_destroy", "symi_workspace_bytes", "symi_last_error",
    "symi_route", "symi_route_bwd", "symi_place", "symi_place_host", "symi_dispatch",
    "symi_dispatch_noalloc", "symi_slot_capacity", "symi_dispatch_capacity", "symi_dispatch_bwd", "symi_expert_fwd",
    "symi_expert_bwd", "symi_combine", "symi_combine_bwd", "symi_adam_to_replicas",
    "symi_expert_bwd_slots", "symi_expert_bwd_active", "symi_adam_to_replicas_active",
    "symi_replica_allreduce", "symi_router_fwd", "symi_router_bwd",
    "symi_grad_source", "symi_collect_grads", "symi_rank_group", "symi_comm_cost",
    "symi_timing_reset", "symi_timing_read", "symi_kernel_count", "symi_kernel_name",
]


class SymiError(RuntimeError):
    pass


class SymiCfg(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in
                ("T", "E", "k", "d", "f", "S_tot", "N", "shard", "dtype", "renorm")]

    @classmethod
    def make(cls, T, E, k, d, f, S_tot, N, shard=0, dtype="bf16", renorm=1):
        return cls(T, E, k, d, f, S_tot, N, shard, {"f32": 0, "bf16": 1}[dtype], int(renorm))

    @property
    def A(self):
        return self.T * self.k

    @property
    def torch_dtype(self):
        return torch.bfloat16 if self.dtype == 1 else torch.float32


CTX_NO_OVERLAP, CTX_NO_SLICING, CTX_TIMING = 1, 2, 4


class SymiCtx:
    """Handle of a symi_ctx (symi_create); `cfg` is the configuration it was created from."""

    def __init__(self, ptr, cfg, flags):
        self.ptr, self.cfg, self.flags = ptr, cfg, flags

    def __getattr__(self, name):          # sizes and dtype read through to the configuration
        if name in ("ptr", "cfg", "flags"):
            raise AttributeError(name)
        return getattr(self.cfg, name)

    def __del__(self):
        try:
            if self.ptr:
                symi_destroy(self)
        except Exception:
            pass


class SymiCostIn(ctypes.Structure):
    _fields_ = [("E", ctypes.c_int), ("N", ctypes.c_int), ("s", ctypes.c_int), ("G", ctypes.c_double),
                ("W", ctypes.c_double), ("O", ctypes.c_double), ("bw_pci", ctypes.c_double),
                ("bw_net", ctypes.c_double)]


class SymiCostOut(ctypes.Structure):
    _fields_ = [(n, ctypes.c_double) for n in (
        "mem_static", "mem_symi", "data_grad_static", "data_weight_static", "data_grad_symi",
        "data_weight_symi", "t_grad_static", "t_weight_static", "t_grad_symi", "t_weight_symi",
        "extra_fraction")]


class SymiAdam(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_float), ("beta1", ctypes.c_float), ("beta2", ctypes.c_float),
                ("eps", ctypes.c_float), ("weight_decay", ctypes.c_float),
                ("grad_scale", ctypes.c_float), ("step", ctypes.c_int)]


def lib_path():
    """The in-tree library; SYMI_LIB names another build of it (A/B measurements)."""
    return os.environ.get("SYMI_LIB") or os.path.join(_HERE, "libsymi.so")


def lib():
    """Loads libsymi.so once; raises if it has not been built."""
    global _LIB
    if _LIB is None:
        path = lib_path()
        if not os.path.exists(path):
            raise SymiError(f"{path} not found: build it with `python -m paper_2504_19925_amd.build`")
        L = ctypes.CDLL(path)
        vp, ip, fp = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p
        cfgp, ctx = ctypes.POINTER(SymiCfg), ctypes.c_void_p
        ci, cf, cd = ctypes.c_int, ctypes.c_float, ctypes.c_double
        sig = {   # name: (argument types, result type)
            "symi_validate": ([cfgp], ci),
            "symi_create": ([cfgp, ctypes.c_uint, ctypes.POINTER(ctypes.c_void_p)], ci),
            "symi_destroy": ([ctx], ci),
            "symi_workspace_bytes": ([cfgp], ctypes.c_size_t),
            "symi_last_error": ([], ctypes.c_char_p),
            "symi_route": ([ctx, fp, ip, fp, ip, vp], ci),
            "symi_route_bwd": ([ctx, fp, ip, fp, fp, fp, vp], ci),
            "symi_place": ([ctx, ip, ip, ip, ip, vp], ci),
            "symi_place_host": ([cfgp, ip, ip, ip, ip], ci),
            "symi_dispatch": ([ctx, vp, ip, ip, ip, ip, ip, ip, ip, vp, vp, vp], ci),
            "symi_dispatch_noalloc": ([ctx, vp, ip, ip, ip, ip, ip, ip, ip, vp, vp], ci),
            "symi_slot_capacity": ([cfgp, cd], ci),
            "symi_dispatch_capacity": ([ctx, ci, vp, ip, ip, ip, ip, ip, ip, ip, vp, vp, vp], ci),
            "symi_dispatch_bwd": ([ctx, vp, ip, vp, vp], ci),
            "symi_expert_fwd": ([ctx, vp, ip, vp, vp, vp, vp, vp, vp, vp], ci),
            "symi_expert_bwd": ([ctx, vp, vp, vp, vp, ip, ip, vp, vp, vp, fp, fp, vp, vp], ci),
            "symi_expert_bwd_slots": ([ctx, vp, vp, vp, vp, ip, ip, vp, vp, vp, fp, fp, vp, vp], ci),
            "symi_expert_bwd_active": ([ctx, vp, vp, vp, vp, ip, ip, vp, vp, vp, fp, fp, vp, vp], ci),
            "symi_replica_allreduce": ([ctx, ip, cf, fp, fp, vp], ci),
            "symi_router_fwd": ([ctx, vp, vp, fp, fp, vp], ci),
            "symi_router_bwd": ([ctx, vp, vp, fp, fp, fp, vp, vp, vp], ci),
            "symi_combine": ([ctx, vp, ip, fp, vp, vp], ci),
            "symi_combine_bwd": ([ctx, vp, vp, ip, fp, vp, fp, vp], ci),
            "symi_adam_to_replicas": ([ctx, ctypes.POINTER(SymiAdam), fp, fp, fp, fp, fp, ip, vp, vp, vp], ci),
            "symi_adam_to_replicas_active": ([ctx, ctypes.POINTER(SymiAdam), fp, fp, fp, fp, fp, ip, ip, ip,
                                              vp, vp, vp], ci),
            "symi_grad_source": ([cfgp, vp, ci, ci], ci),
            "symi_collect_grads": ([cfgp, vp, ci, vp, vp, vp, ci], ci),
            "symi_rank_group": ([ci, ci, ci], ci),
            "symi_comm_cost": ([ctypes.POINTER(SymiCostIn), ctypes.POINTER(SymiCostOut)], ci),
            "symi_timing_reset": ([ctx], ci),
            "symi_timing_read": ([ctx, ci, ctypes.POINTER(cd), ctypes.POINTER(ci)], ci),
            "symi_kernel_count": ([], ci),
            "symi_kernel_name": ([ci], ctypes.c_char_p),
        }
        for name, (args, res) in sig.items():
            fn = getattr(L, name)
            fn.argtypes = args
            fn.restype = res
        _LIB = L
    return _LIB


def symi_last_error():
    return lib().symi_last_error().decode()


def _check(rc, who):
    if rc != 0:
        raise SymiError(f"{who} failed ({rc}): {symi_last_error()}")


def _dev(t, dtype, name, numel=None):
    if not isinstance(t, torch.Tensor):
        raise SymiError(f"{name}: expected a torch tensor")
    if not t.is_cuda:
        raise SymiError(f"{name}: expected a GPU tensor")
    if t.dtype != dtype:
        raise SymiError(f"{name}: expected dtype {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise SymiError(f"{name}: must be contiguous")
    if numel is not None and t.numel() < numel:
        raise SymiError(f"{name}: needs at least {numel} elements, has {t.numel()}")
    return ctypes.c_void_p(t.data_ptr())


def _host_i32(t, name, numel):
    if not isinstance(t, torch.Tensor) or t.is_cuda or t.dtype != I32 or not t.is_contiguous() or t.numel() < numel:
        raise SymiError(f"{name}: expected a contiguous CPU int32 tensor with >= {numel} elements")
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


I32, F32 = torch.int32, torch.float32


def symi_create(cfg, flags=0):
    out = ctypes.c_void_p()
    _check(lib().symi_create(ctypes.byref(cfg), int(flags), ctypes.byref(out)), "symi_create")
    return SymiCtx(out, cfg, int(flags))


def symi_destroy(ctx):
    ptr, ctx.ptr = ctx.ptr, None
    if ptr:
        _check(lib().symi_destroy(ptr), "symi_destroy")


def symi_timing_reset(ctx):
    _check(lib().symi_timing_reset(ctx.ptr), "symi_timing_reset")


def symi_timing_read(ctx, kernel_id):
    """(total milliseconds, launches) of one kernel id since the last reset."""
    ms, n = ctypes.c_double(0.0), ctypes.c_int(0)
    _check(lib().symi_timing_read(ctx.ptr, int(kernel_id), ctypes.byref(ms), ctypes.byref(n)),
           "symi_timing_read")
    return ms.value, n.value


def symi_kernel_count():
    return lib().symi_kernel_count()


def symi_kernel_name(kernel_id):
    return lib().symi_kernel_name(int(kernel_id)).decode()


def _cfg_of(x):
    """Host functions take the configuration; a context stands for the one it was created from."""
    return x.cfg if isinstance(x, SymiCtx) else x


def symi_validate(cfg):
    return lib().symi_validate(ctypes.byref(_cfg_of(cfg)))


def symi_workspace_bytes(cfg):
    return lib().symi_workspace_bytes(ctypes.byref(_cfg_of(cfg)))


def symi_route(ctx, logits, idx, gate, hist):
    _check(lib().symi_route(ctx.ptr, _dev(logits, F32, "logits", ctx.T * ctx.E),
                            _dev(idx, I32, "idx", ctx.A), _dev(gate, F32, "gate", ctx.A),
                            _dev(hist, I32, "hist", ctx.E), _stream()), "symi_route")


def symi_route_bwd(ctx, logits, idx, gate, dgate, dlogits):
    _check(lib().symi_route_bwd(ctx.ptr, _dev(logits, F32, "logits", ctx.T * ctx.E),
                                _dev(idx, I32, "idx", ctx.A), _dev(gate, F32, "gate", ctx.A),
                                _dev(dgate, F32, "dgate", ctx.A),
                                _dev(dlogits, F32, "dlogits", ctx.T * ctx.E), _stream()),
           "symi_route_bwd")


def symi_place(ctx, popularity, counts, placement, first_slot):
    _check(lib().symi_place(ctx.ptr, _dev(popularity, I32, "popularity", ctx.E),
                            _dev(counts, I32, "counts", ctx.E),
                            _dev(placement, I32, "placement", ctx.S_tot),
                            _dev(first_slot, I32, "first_slot", ctx.E + 1), _stream()), "symi_place")


def symi_place_host(cfg, popularity, counts, placement, first_slot):
    cfg = _cfg_of(cfg)
    _check(lib().symi_place_host(ctypes.byref(cfg), _host_i32(popularity, "popularity", cfg.E),
                                 _host_i32(counts, "counts", cfg.E),
                                 _host_i32(placement, "placement", cfg.S_tot),
                                 _host_i32(first_slot, "first_slot", cfg.E + 1)), "symi_place_host")


def symi_dispatch(ctx, X, idx, hist, counts, first_slot, row_of_assign, assign_of_row,
                  slot_offsets, Xp, ws):
    dt = ctx.torch_dtype
    _check(lib().symi_dispatch(
        ctx.ptr, _dev(X, dt, "X", ctx.T * ctx.d), _dev(idx, I32, "idx", ctx.A),
        _dev(hist, I32, "hist", ctx.E), _dev(counts, I32, "counts", ctx.E),
        _dev(first_slot, I32, "first_slot", ctx.E + 1),
        _dev(row_of_assign, I32, "row_of_assign", ctx.A),
        _dev(assign_of_row, I32, "assign_of_row", ctx.A),
        _dev(slot_offsets, I32, "slot_offsets", ctx.S_tot + 1), _dev(Xp, dt, "Xp", ctx.A * ctx.d),
        _dev(ws, torch.uint8, "ws", symi_workspace_bytes(ctx.cfg)), _stream()), "symi_dispatch")


def symi_dispatch_noalloc(ctx, X, idx, hist, counts, first_slot, row_of_assign, assign_of_row,
                          slot_offsets, Xp):
    dt = ctx.torch_dtype
    _check(lib().symi_dispatch_noalloc(
        ctx.ptr, _dev(X, dt, "X", ctx.T * ctx.d), _dev(idx, I32, "idx", ctx.A),
        _dev(hist, I32, "hist", ctx.E), _dev(counts, I32, "counts", ctx.E),
        _dev(first_slot, I32, "first_slot", ctx.E + 1),
        _dev(row_of_assign, I32, "row_of_assign", ctx.A),
        _dev(assign_of_row, I32, "assign_of_row", ctx.A),
        _dev(slot_offsets, I32, "slot_offsets", ctx.S_tot + 1), _dev(Xp, dt, "Xp", ctx.A * ctx.d),
        _stream()), "symi_dispatch_noalloc")


def symi_slot_capacity(cfg, capacity_factor):
    cfg = _cfg_of(cfg)
    rc = lib().symi_slot_capacity(ctypes.byref(cfg), float(capacity_factor))
    if rc < 0:
        _check(rc, "symi_slot_capacity")
    return rc


def symi_dispatch_capacity(ctx, slot_capacity, X, idx, hist, counts, first_slot, row_of_assign,
                           assign_of_row, slot_offsets, Xp, ws):
    dt = ctx.torch_dtype
    _check(lib().symi_dispatch_capacity(
        ctx.ptr, int(slot_capacity), _dev(X, dt, "X", ctx.T * ctx.d),
        _dev(idx, I32, "idx", ctx.A), _dev(hist, I32, "hist", ctx.E),
        _dev(counts, I32, "counts", ctx.E), _dev(first_slot, I32, "first_slot", ctx.E + 1),
        _dev(row_of_assign, I32, "row_of_assign", ctx.A),
        _dev(assign_of_row, I32, "assign_of_row", ctx.A),
        _dev(slot_offsets, I32, "slot_offsets", ctx.S_tot + 1), _dev(Xp, dt, "Xp", ctx.A * ctx.d),
        _dev(ws, torch.uint8, "ws", symi_workspace_bytes(ctx.cfg)), _stream()), "symi_dispatch_capacity")


def symi_grad_source(cfg, placement, exp_id, rank):
    cfg = _cfg_of(cfg)
    rc = lib().symi_grad_source(ctypes.byref(cfg), _host_i32(placement, "placement", cfg.S_tot),
                                int(exp_id), int(rank))
    if rc < 0:
        _check(rc, "symi_grad_source")
    return rc


def symi_collect_grads(cfg, placement, rank, recv_src, send_offsets, send_dst):
    cfg = _cfg_of(cfg)
    rc = lib().symi_collect_grads(ctypes.byref(cfg), _host_i32(placement, "placement", cfg.S_tot), int(rank),
                                  _host_i32(recv_src, "recv_src", cfg.E),
                                  _host_i32(send_offsets, "send_offsets", cfg.E + 1),
                                  _host_i32(send_dst, "send_dst", 0), int(send_dst.numel()))
    if rc < 0:
        _check(rc, "symi_collect_grads")
    return rc


def symi_rank_group(N, first_rank, last_rank):
    rc = lib().symi_rank_group(int(N), int(first_rank), int(last_rank))
    if rc < 0:
        _check(rc, "symi_rank_group")
    return rc


def symi_comm_cost(E, N, s, G, W, O, bw_pci, bw_net):
    cin = SymiCostIn(int(E), int(N), int(s), float(G), float(W), float(O), float(bw_pci), float(bw_net))
    out = SymiCostOut()
    _check(lib().symi_comm_cost(ctypes.byref(cin), ctypes.byref(out)), "symi_comm_cost")
    return {n: getattr(out, n) for n, _ in SymiCostOut._fields_}


def symi_dispatch_bwd(ctx, dXp, row_of_assign, dX):
    dt = ctx.torch_dtype
    _check(lib().symi_dispatch_bwd(ctx.ptr, _dev(dXp, dt, "dXp", ctx.A * ctx.d),
                                   _dev(row_of_assign, I32, "row_of_assign", ctx.A),
                                   _dev(dX, dt, "dX", ctx.T * ctx.d), _stream()), "symi_dispatch_bwd")


def symi_expert_fwd(ctx, Xp, slot_offsets, W1_slots, W2_slots, UV, H, Yp, ws):
    dt = ctx.torch_dtype
    nw = ctx.S_tot * ctx.d * ctx.f
    _check(lib().symi_expert_fwd(
        ctx.ptr, _dev(Xp, dt, "Xp", ctx.A * ctx.d),
        _dev(slot_offsets, I32, "slot_offsets", ctx.S_tot + 1),
        _dev(W1_slots, dt, "W1_slots", 2 * nw), _dev(W2_slots, dt, "W2_slots", nw),
        _dev(UV, dt, "UV", ctx.A * 2 * ctx.f), _dev(H, dt, "H", ctx.A * ctx.f),
        _dev(Yp, dt, "Yp", ctx.A * ctx.d), _dev(ws, torch.uint8, "ws", symi_workspace_bytes(ctx.cfg)),
        _stream()), "symi_expert_fwd")


def _expert_bwd_class(name, ctx, dYp, Xp, UV, H, slot_offsets, first_slot, W1_slots, W2_slots, dXp,
                      dW1_class, dW2_class, ws):
    dt = ctx.torch_dtype
    nw = ctx.S_tot * ctx.d * ctx.f
    ne = ctx.E * ctx.d * ctx.f
    _check(getattr(lib(), name)(
        ctx.ptr, _dev(dYp, dt, "dYp", ctx.A * ctx.d), _dev(Xp, dt, "Xp", ctx.A * ctx.d),
        _dev(UV, dt, "UV", ctx.A * 2 * ctx.f), _dev(H, dt, "H", ctx.A * ctx.f),
        _dev(slot_offsets, I32, "slot_offsets", ctx.S_tot + 1),
        _dev(first_slot, I32, "first_slot", ctx.E + 1), _dev(W1_slots, dt, "W1_slots", 2 * nw),
        _dev(W2_slots, dt, "W2_slots", nw), _dev(dXp, dt, "dXp", ctx.A * ctx.d),
        _dev(dW1_class, F32, "dW1_class", 2 * ne), _dev(dW2_class, F32, "dW2_class", ne),
        _dev(ws, torch.uint8, "ws", symi_workspace_bytes(ctx.cfg)), _stream()), name)


def symi_expert_bwd(ctx, dYp, Xp, UV, H, slot_offsets, first_slot, W1_slots, W2_slots, dXp,
                    dW1_class, dW2_class, ws):
    _expert_bwd_class("symi_expert_bwd", ctx, dYp, Xp, UV, H, slot_offsets, first_slot, W1_slots,
                      W2_slots, dXp, dW1_class, dW2_class, ws)


def symi_expert_bwd_active(ctx, dYp, Xp, UV, H, slot_offsets, first_slot, W1_slots, W2_slots, dXp,
                           dW1_class, dW2_class, ws):
    _expert_bwd_class("symi_expert_bwd_active", ctx, dYp, Xp, UV, H, slot_offsets, first_slot,
                      W1_slots, W2_slots, dXp, dW1_class, dW2_class, ws)


def symi_expert_bwd_slots(ctx, dYp, Xp, UV, H, slot_offsets, first_slot, W1_slots, W2_slots, dXp,
                          dW1_slot, dW2_slot, ws):
    dt = ctx.torch_dtype
    nw = ctx.S_tot * ctx.d * ctx.f
    _check(lib().symi_expert_bwd_slots(
        ctx.ptr, _dev(dYp, dt, "dYp", ctx.A * ctx.d), _dev(Xp, dt, "Xp", ctx.A * ctx.d),
        _dev(UV, dt, "UV", ctx.A * 2 * ctx.f), _dev(H, dt, "H", ctx.A * ctx.f),
        _dev(slot_offsets, I32, "slot_offsets", ctx.S_tot + 1),
        _dev(first_slot, I32, "first_slot", ctx.E + 1), _dev(W1_slots, dt, "W1_slots", 2 * nw),
        _dev(W2_slots, dt, "W2_slots", nw), _dev(dXp, dt, "dXp", ctx.A * ctx.d),
        _dev(dW1_slot, F32, "dW1_slot", 2 * nw), _dev(dW2_slot, F32, "dW2_slot", nw),
        _dev(ws, torch.uint8, "ws", symi_workspace_bytes(ctx.cfg)), _stream()), "symi_expert_bwd_slots")


def symi_replica_allreduce(ctx, first_slot, scale, dW1_slot, dW2_slot):
    nw = ctx.S_tot * ctx.d * ctx.f
    _check(lib().symi_replica_allreduce(
        ctx.ptr, _dev(first_slot, I32, "first_slot", ctx.E + 1), ctypes.c_float(scale),
        _dev(dW1_slot, F32, "dW1_slot", 2 * nw), _dev(dW2_slot, F32, "dW2_slot", nw), _stream()),
        "symi_replica_allreduce")


def symi_router_fwd(ctx, X, Wr, b, logits):
    dt = ctx.torch_dtype
    _check(lib().symi_router_fwd(
        ctx.ptr, _dev(X, dt, "X", ctx.T * ctx.d), _dev(Wr, dt, "Wr", ctx.E * ctx.d),
        None if b is None else _dev(b, F32, "b", ctx.E), _dev(logits, F32, "logits", ctx.T * ctx.E),
        _stream()), "symi_router_fwd")


def symi_router_bwd(ctx, X, Wr, dlogits, dWr, db, dX, ws):
    dt = ctx.torch_dtype
    _check(lib().symi_router_bwd(
        ctx.ptr, _dev(X, dt, "X", ctx.T * ctx.d), _dev(Wr, dt, "Wr", ctx.E * ctx.d),
        _dev(dlogits, F32, "dlogits", ctx.T * ctx.E), _dev(dWr, F32, "dWr", ctx.E * ctx.d),
        None if db is None else _dev(db, F32, "db", ctx.E), _dev(dX, dt, "dX", ctx.T * ctx.d),
        _dev(ws, torch.uint8, "ws", symi_workspace_bytes(ctx.cfg)), _stream()), "symi_router_bwd")


def symi_combine(ctx, Yp, row_of_assign, gate, Y):
    dt = ctx.torch_dtype
    _check(lib().symi_combine(ctx.ptr, _dev(Yp, dt, "Yp", ctx.A * ctx.d),
                              _dev(row_of_assign, I32, "row_of_assign", ctx.A),
                              _dev(gate, F32, "gate", ctx.A), _dev(Y, dt, "Y", ctx.T * ctx.d),
                              _stream()), "symi_combine")


def symi_combine_bwd(ctx, dY, Yp, row_of_assign, gate, dYp, dgate):
    dt = ctx.torch_dtype
    _check(lib().symi_combine_bwd(
        ctx.ptr, _dev(dY, dt, "dY", ctx.T * ctx.d), _dev(Yp, dt, "Yp", ctx.A * ctx.d),
        _dev(row_of_assign, I32, "row_of_assign", ctx.A), _dev(gate, F32, "gate", ctx.A),
        _dev(dYp, dt, "dYp", ctx.A * ctx.d), _dev(dgate, F32, "dgate", ctx.A), _stream()),
        "symi_combine_bwd")


def symi_adam_to_replicas(ctx, hp, dW1_class, dW2_class, master_w, m, v, first_slot_next,
                          W1_slots, W2_slots):
    dt = ctx.torch_dtype
    ne = ctx.E * ctx.d * ctx.f
    nw = ctx.S_tot * ctx.d * ctx.f
    per = ctx.E * (3 * ctx.d * ctx.f // ctx.N)
    _check(lib().symi_adam_to_replicas(
        ctx.ptr, ctypes.byref(hp), _dev(dW1_class, F32, "dW1_class", 2 * ne),
        _dev(dW2_class, F32, "dW2_class", ne), _dev(master_w, F32, "master_w", per),
        _dev(m, F32, "m", per), _dev(v, F32, "v", per),
        _dev(first_slot_next, I32, "first_slot_next", ctx.E + 1),
        _dev(W1_slots, dt, "W1_slots", 2 * nw), _dev(W2_slots, dt, "W2_slots", nw), _stream()),
        "symi_adam_to_replicas")


def symi_adam_to_replicas_active(ctx, hp, dW1_class, dW2_class, master_w, m, v, slot_offsets,
                                 first_slot, first_slot_next, W1_slots, W2_slots):
    dt = ctx.torch_dtype
    ne = ctx.E * ctx.d * ctx.f
    nw = ctx.S_tot * ctx.d * ctx.f
    per = ctx.E * (3 * ctx.d * ctx.f // ctx.N)
    _check(lib().symi_adam_to_replicas_active(
        ctx.ptr, ctypes.byref(hp), _dev(dW1_class, F32, "dW1_class", 2 * ne),
        _dev(dW2_class, F32, "dW2_class", ne), _dev(master_w, F32, "master_w", per),
        _dev(m, F32, "m", per), _dev(v, F32, "v", per),
        _dev(slot_offsets, I32, "slot_offsets", ctx.S_tot + 1),
        _dev(first_slot, I32, "first_slot", ctx.E + 1),
        _dev(first_slot_next, I32, "first_slot_next", ctx.E + 1),
        _dev(W1_slots, dt, "W1_slots", 2 * nw), _dev(W2_slots, dt, "W2_slots", nw), _stream()),
        "symi_adam_to_replicas_active")
