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
    "symi_validate", "symi_workspace_bytes", "symi_last_error", "symi_route", "symi_route_bwd",
    "symi_place", "symi_place_host", "symi_dispatch", "symi_slot_capacity",
    "symi_dispatch_capacity", "symi_dispatch_bwd", "symi_expert_fwd",
    "symi_expert_bwd", "symi_combine", "symi_combine_bwd", "symi_adam_to_replicas",
    "symi_timing_enable", "symi_timing_reset", "symi_timing_read", "symi_kernel_count",
    "symi_kernel_name", "symi_expert_bwd_slots", "symi_expert_bwd_active", "symi_adam_to_replicas_active", "symi_set_overlap", "symi_set_slicing", "symi_replica_allreduce", "symi_router_fwd", "symi_router_bwd",
    "symi_grad_source", "symi_collect_grads", "symi_rank_group", "symi_comm_cost",
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
    return os.path.join(_HERE, "libsymi.so")


def lib():
    """Loads libsymi.so once; raises if it has not been built."""
    global _LIB
    if _LIB is None:
        path = lib_path()
        if not os.path.exists(path):
            raise SymiError(f"{path} not found: build it with `python -m paper_2504_19925_amd.build`")
        L = ctypes.CDLL(path)
        vp, ip, fp = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p
        cfgp = ctypes.POINTER(SymiCfg)
        sig = {
            "symi_validate": [cfgp],
            "symi_route": [cfgp, fp, ip, fp, ip, vp],
            "symi_route_bwd": [cfgp, fp, ip, fp, fp, fp, vp],
            "symi_place": [cfgp, ip, ip, ip, ip, vp],
            "symi_place_host": [cfgp, ip, ip, ip, ip],
            "symi_dispatch": [cfgp, vp, ip, ip, ip, ip, ip, ip, ip, vp, vp, vp],
            "symi_slot_capacity": [cfgp, ctypes.c_double],
            "symi_dispatch_capacity": [cfgp, ctypes.c_int, vp, ip, ip, ip, ip, ip, ip, ip, vp, vp, vp],
            "symi_dispatch_bwd": [cfgp, vp, ip, vp, vp],
            "symi_expert_fwd": [cfgp, vp, ip, vp, vp, vp, vp, vp, vp, vp],
            "symi_expert_bwd": [cfgp, vp, vp, vp, vp, ip, ip, vp, vp, vp, fp, fp, vp, vp],
            "symi_expert_bwd_slots": [cfgp, vp, vp, vp, vp, ip, ip, vp, vp, vp, fp, fp, vp, vp],
            "symi_expert_bwd_active": [cfgp, vp, vp, vp, vp, ip, ip, vp, vp, vp, fp, fp, vp, vp],
            "symi_replica_allreduce": [cfgp, ip, ctypes.c_float, fp, fp, vp],
            "symi_router_fwd": [cfgp, vp, vp, fp, fp, vp],
            "symi_router_bwd": [cfgp, vp, vp, fp, fp, fp, vp, vp, vp],
            "symi_combine": [cfgp, vp, ip, fp, vp, vp],
            "symi_combine_bwd": [cfgp, vp, vp, ip, fp, vp, fp, vp],
            "symi_adam_to_replicas": [cfgp, ctypes.POINTER(SymiAdam), fp, fp, fp, fp, fp, ip, vp, vp, vp],
            "symi_adam_to_replicas_active": [cfgp, ctypes.POINTER(SymiAdam), fp, fp, fp, fp, fp, ip, ip, ip,
                                             vp, vp, vp],
        }
        for name, args in sig.items():
            fn = getattr(L, name)
            fn.argtypes = args
            fn.restype = ctypes.c_int
        L.symi_grad_source.argtypes = [cfgp, ctypes.c_void_p, ctypes.c_int, ctypes.c_int]
        L.symi_collect_grads.argtypes = [cfgp, ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p,
                                         ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int]
        L.symi_rank_group.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int]
        L.symi_comm_cost.argtypes = [ctypes.POINTER(SymiCostIn), ctypes.POINTER(SymiCostOut)]
        for name in ("symi_expert_bwd_slots", "symi_set_overlap", "symi_set_slicing", "symi_replica_allreduce", "symi_router_fwd", "symi_router_bwd",
    "symi_grad_source", "symi_collect_grads", "symi_rank_group", "symi_comm_cost"):
            getattr(L, name).restype = ctypes.c_int
        L.symi_workspace_bytes.argtypes = [cfgp]
        L.symi_workspace_bytes.restype = ctypes.c_size_t
        L.symi_last_error.argtypes = []
        L.symi_last_error.restype = ctypes.c_char_p
        L.symi_set_overlap.argtypes = [ctypes.c_int]
        L.symi_set_overlap.restype = ctypes.c_int
        L.symi_set_slicing.argtypes = [ctypes.c_int]
        L.symi_set_slicing.restype = ctypes.c_int
        L.symi_timing_enable.argtypes = [ctypes.c_int]
        L.symi_timing_reset.argtypes = []
        L.symi_timing_read.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_double),
                                       ctypes.POINTER(ctypes.c_int)]
        L.symi_kernel_count.argtypes = []
        L.symi_kernel_name.argtypes = [ctypes.c_int]
        L.symi_kernel_name.restype = ctypes.c_char_p
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
    if t.is_cuda or t.dtype != torch.int32 or not t.is_contiguous() or t.numel() < numel:
        raise SymiError(f"{name}: expected a contiguous CPU int32 tensor of >= {numel} elements")
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


I32, F32 = torch.int32, torch.float32


def symi_timing_enable(on):
    _check(lib().symi_timing_enable(int(bool(on))), "symi_timing_enable")


def symi_timing_reset():
    _check(lib().symi_timing_reset(), "symi_timing_reset")


def symi_timing_read(kernel_id):
    """(total milliseconds, launches) of one kernel id since the last reset."""
    ms, n = ctypes.c_double(0.0), ctypes.c_int(0)
    _check(lib().symi_timing_read(int(kernel_id), ctypes.byref(ms), ctypes.byref(n)),
           "symi_timing_read")
    return ms.value, n.value


def symi_kernel_count():
    return lib().symi_kernel_count()


def symi_kernel_name(kernel_id):
    return lib().symi_kernel_name(int(kernel_id)).decode()


def symi_validate(cfg):
    return lib().symi_validate(ctypes.byref(cfg))


def symi_workspace_bytes(cfg):
    return lib().symi_workspace_bytes(ctypes.byref(cfg))


def symi_route(cfg, logits, idx, gate, hist):
    _check(lib().symi_route(ctypes.byref(cfg), _dev(logits, F32, "logits", cfg.T * cfg.E),
                            _dev(idx, I32, "idx", cfg.A), _dev(gate, F32, "gate", cfg.A),
                            _dev(hist, I32, "hist", cfg.E), _stream()), "symi_route")


def symi_route_bwd(cfg, logits, idx, gate, dgate, dlogits):
    _check(lib().symi_route_bwd(ctypes.byref(cfg), _dev(logits, F32, "logits", cfg.T * cfg.E),
                                _dev(idx, I32, "idx", cfg.A), _dev(gate, F32, "gate", cfg.A),
                                _dev(dgate, F32, "dgate", cfg.A),
                                _dev(dlogits, F32, "dlogits", cfg.T * cfg.E), _stream()),
           "symi_route_bwd")


def symi_place(cfg, popularity, counts, placement, first_slot):
    _check(lib().symi_place(ctypes.byref(cfg), _dev(popularity, I32, "popularity", cfg.E),
                            _dev(counts, I32, "counts", cfg.E),
                            _dev(placement, I32, "placement", cfg.S_tot),
                            _dev(first_slot, I32, "first_slot", cfg.E + 1), _stream()), "symi_place")


def symi_place_host(cfg, popularity, counts, placement, first_slot):
    _check(lib().symi_place_host(ctypes.byref(cfg), _host_i32(popularity, "popularity", cfg.E),
                                 _host_i32(counts, "counts", cfg.E),
                                 _host_i32(placement, "placement", cfg.S_tot),
                                 _host_i32(first_slot, "first_slot", cfg.E + 1)), "symi_place_host")


def symi_dispatch(cfg, X, idx, hist, counts, first_slot, row_of_assign, assign_of_row,
                  slot_offsets, Xp, ws):
    dt = cfg.torch_dtype
    _check(lib().symi_dispatch(
        ctypes.byref(cfg), _dev(X, dt, "X", cfg.T * cfg.d), _dev(idx, I32, "idx", cfg.A),
        _dev(hist, I32, "hist", cfg.E), _dev(counts, I32, "counts", cfg.E),
        _dev(first_slot, I32, "first_slot", cfg.E + 1),
        _dev(row_of_assign, I32, "row_of_assign", cfg.A),
        _dev(assign_of_row, I32, "assign_of_row", cfg.A),
        _dev(slot_offsets, I32, "slot_offsets", cfg.S_tot + 1), _dev(Xp, dt, "Xp", cfg.A * cfg.d),
        _dev(ws, torch.uint8, "ws", symi_workspace_bytes(cfg)), _stream()), "symi_dispatch")


def symi_slot_capacity(cfg, capacity_factor):
    rc = lib().symi_slot_capacity(ctypes.byref(cfg), float(capacity_factor))
    if rc < 0:
        _check(rc, "symi_slot_capacity")
    return rc


def symi_dispatch_capacity(cfg, slot_capacity, X, idx, hist, counts, first_slot, row_of_assign,
                           assign_of_row, slot_offsets, Xp, ws):
    dt = cfg.torch_dtype
    _check(lib().symi_dispatch_capacity(
        ctypes.byref(cfg), int(slot_capacity), _dev(X, dt, "X", cfg.T * cfg.d),
        _dev(idx, I32, "idx", cfg.A), _dev(hist, I32, "hist", cfg.E),
        _dev(counts, I32, "counts", cfg.E), _dev(first_slot, I32, "first_slot", cfg.E + 1),
        _dev(row_of_assign, I32, "row_of_assign", cfg.A),
        _dev(assign_of_row, I32, "assign_of_row", cfg.A),
        _dev(slot_offsets, I32, "slot_offsets", cfg.S_tot + 1), _dev(Xp, dt, "Xp", cfg.A * cfg.d),
        _dev(ws, torch.uint8, "ws", symi_workspace_bytes(cfg)), _stream()), "symi_dispatch_capacity")


def _host_i32(t, name, numel):
    if not isinstance(t, torch.Tensor) or t.is_cuda or t.dtype != I32 or not t.is_contiguous() or t.numel() < numel:
        raise SymiError(f"{name}: expected a contiguous CPU int32 tensor with >= {numel} elements")
    return ctypes.c_void_p(t.data_ptr())


def symi_grad_source(cfg, placement, exp_id, rank):
    rc = lib().symi_grad_source(ctypes.byref(cfg), _host_i32(placement, "placement", cfg.S_tot),
                                int(exp_id), int(rank))
    if rc < 0:
        _check(rc, "symi_grad_source")
    return rc


def symi_collect_grads(cfg, placement, rank, recv_src, send_offsets, send_dst):
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


def symi_dispatch_bwd(cfg, dXp, row_of_assign, dX):
    dt = cfg.torch_dtype
    _check(lib().symi_dispatch_bwd(ctypes.byref(cfg), _dev(dXp, dt, "dXp", cfg.A * cfg.d),
                                   _dev(row_of_assign, I32, "row_of_assign", cfg.A),
                                   _dev(dX, dt, "dX", cfg.T * cfg.d), _stream()), "symi_dispatch_bwd")


def symi_expert_fwd(cfg, Xp, slot_offsets, W1_slots, W2_slots, UV, H, Yp, ws):
    dt = cfg.torch_dtype
    nw = cfg.S_tot * cfg.d * cfg.f
    _check(lib().symi_expert_fwd(
        ctypes.byref(cfg), _dev(Xp, dt, "Xp", cfg.A * cfg.d),
        _dev(slot_offsets, I32, "slot_offsets", cfg.S_tot + 1),
        _dev(W1_slots, dt, "W1_slots", 2 * nw), _dev(W2_slots, dt, "W2_slots", nw),
        _dev(UV, dt, "UV", cfg.A * 2 * cfg.f), _dev(H, dt, "H", cfg.A * cfg.f),
        _dev(Yp, dt, "Yp", cfg.A * cfg.d), _dev(ws, torch.uint8, "ws", symi_workspace_bytes(cfg)),
        _stream()), "symi_expert_fwd")


def _expert_bwd_class(name, cfg, dYp, Xp, UV, H, slot_offsets, first_slot, W1_slots, W2_slots, dXp,
                      dW1_class, dW2_class, ws):
    dt = cfg.torch_dtype
    nw = cfg.S_tot * cfg.d * cfg.f
    ne = cfg.E * cfg.d * cfg.f
    _check(getattr(lib(), name)(
        ctypes.byref(cfg), _dev(dYp, dt, "dYp", cfg.A * cfg.d), _dev(Xp, dt, "Xp", cfg.A * cfg.d),
        _dev(UV, dt, "UV", cfg.A * 2 * cfg.f), _dev(H, dt, "H", cfg.A * cfg.f),
        _dev(slot_offsets, I32, "slot_offsets", cfg.S_tot + 1),
        _dev(first_slot, I32, "first_slot", cfg.E + 1), _dev(W1_slots, dt, "W1_slots", 2 * nw),
        _dev(W2_slots, dt, "W2_slots", nw), _dev(dXp, dt, "dXp", cfg.A * cfg.d),
        _dev(dW1_class, F32, "dW1_class", 2 * ne), _dev(dW2_class, F32, "dW2_class", ne),
        _dev(ws, torch.uint8, "ws", symi_workspace_bytes(cfg)), _stream()), name)


def symi_expert_bwd(cfg, dYp, Xp, UV, H, slot_offsets, first_slot, W1_slots, W2_slots, dXp,
                    dW1_class, dW2_class, ws):
    _expert_bwd_class("symi_expert_bwd", cfg, dYp, Xp, UV, H, slot_offsets, first_slot, W1_slots,
                      W2_slots, dXp, dW1_class, dW2_class, ws)


def symi_expert_bwd_active(cfg, dYp, Xp, UV, H, slot_offsets, first_slot, W1_slots, W2_slots, dXp,
                           dW1_class, dW2_class, ws):
    _expert_bwd_class("symi_expert_bwd_active", cfg, dYp, Xp, UV, H, slot_offsets, first_slot,
                      W1_slots, W2_slots, dXp, dW1_class, dW2_class, ws)


def symi_expert_bwd_slots(cfg, dYp, Xp, UV, H, slot_offsets, first_slot, W1_slots, W2_slots, dXp,
                          dW1_slot, dW2_slot, ws):
    dt = cfg.torch_dtype
    nw = cfg.S_tot * cfg.d * cfg.f
    _check(lib().symi_expert_bwd_slots(
        ctypes.byref(cfg), _dev(dYp, dt, "dYp", cfg.A * cfg.d), _dev(Xp, dt, "Xp", cfg.A * cfg.d),
        _dev(UV, dt, "UV", cfg.A * 2 * cfg.f), _dev(H, dt, "H", cfg.A * cfg.f),
        _dev(slot_offsets, I32, "slot_offsets", cfg.S_tot + 1),
        _dev(first_slot, I32, "first_slot", cfg.E + 1), _dev(W1_slots, dt, "W1_slots", 2 * nw),
        _dev(W2_slots, dt, "W2_slots", nw), _dev(dXp, dt, "dXp", cfg.A * cfg.d),
        _dev(dW1_slot, F32, "dW1_slot", 2 * nw), _dev(dW2_slot, F32, "dW2_slot", nw),
        _dev(ws, torch.uint8, "ws", symi_workspace_bytes(cfg)), _stream()), "symi_expert_bwd_slots")


def symi_set_overlap(on):
    lib().symi_set_overlap(1 if on else 0)


def symi_set_slicing(on):
    lib().symi_set_slicing(1 if on else 0)


def symi_replica_allreduce(cfg, first_slot, scale, dW1_slot, dW2_slot):
    nw = cfg.S_tot * cfg.d * cfg.f
    _check(lib().symi_replica_allreduce(
        ctypes.byref(cfg), _dev(first_slot, I32, "first_slot", cfg.E + 1), ctypes.c_float(scale),
        _dev(dW1_slot, F32, "dW1_slot", 2 * nw), _dev(dW2_slot, F32, "dW2_slot", nw), _stream()),
        "symi_replica_allreduce")


def symi_router_fwd(cfg, X, Wr, b, logits):
    dt = cfg.torch_dtype
    _check(lib().symi_router_fwd(
        ctypes.byref(cfg), _dev(X, dt, "X", cfg.T * cfg.d), _dev(Wr, dt, "Wr", cfg.E * cfg.d),
        None if b is None else _dev(b, F32, "b", cfg.E), _dev(logits, F32, "logits", cfg.T * cfg.E),
        _stream()), "symi_router_fwd")


def symi_router_bwd(cfg, X, Wr, dlogits, dWr, db, dX, ws):
    dt = cfg.torch_dtype
    _check(lib().symi_router_bwd(
        ctypes.byref(cfg), _dev(X, dt, "X", cfg.T * cfg.d), _dev(Wr, dt, "Wr", cfg.E * cfg.d),
        _dev(dlogits, F32, "dlogits", cfg.T * cfg.E), _dev(dWr, F32, "dWr", cfg.E * cfg.d),
        None if db is None else _dev(db, F32, "db", cfg.E), _dev(dX, dt, "dX", cfg.T * cfg.d),
        _dev(ws, torch.uint8, "ws", symi_workspace_bytes(cfg)), _stream()), "symi_router_bwd")


def symi_combine(cfg, Yp, row_of_assign, gate, Y):
    dt = cfg.torch_dtype
    _check(lib().symi_combine(ctypes.byref(cfg), _dev(Yp, dt, "Yp", cfg.A * cfg.d),
                              _dev(row_of_assign, I32, "row_of_assign", cfg.A),
                              _dev(gate, F32, "gate", cfg.A), _dev(Y, dt, "Y", cfg.T * cfg.d),
                              _stream()), "symi_combine")


def symi_combine_bwd(cfg, dY, Yp, row_of_assign, gate, dYp, dgate):
    dt = cfg.torch_dtype
    _check(lib().symi_combine_bwd(
        ctypes.byref(cfg), _dev(dY, dt, "dY", cfg.T * cfg.d), _dev(Yp, dt, "Yp", cfg.A * cfg.d),
        _dev(row_of_assign, I32, "row_of_assign", cfg.A), _dev(gate, F32, "gate", cfg.A),
        _dev(dYp, dt, "dYp", cfg.A * cfg.d), _dev(dgate, F32, "dgate", cfg.A), _stream()),
        "symi_combine_bwd")


def symi_adam_to_replicas(cfg, hp, dW1_class, dW2_class, master_w, m, v, first_slot_next,
                          W1_slots, W2_slots):
    dt = cfg.torch_dtype
    ne = cfg.E * cfg.d * cfg.f
    nw = cfg.S_tot * cfg.d * cfg.f
    per = cfg.E * (3 * cfg.d * cfg.f // cfg.N)
    _check(lib().symi_adam_to_replicas(
        ctypes.byref(cfg), ctypes.byref(hp), _dev(dW1_class, F32, "dW1_class", 2 * ne),
        _dev(dW2_class, F32, "dW2_class", ne), _dev(master_w, F32, "master_w", per),
        _dev(m, F32, "m", per), _dev(v, F32, "v", per),
        _dev(first_slot_next, I32, "first_slot_next", cfg.E + 1),
        _dev(W1_slots, dt, "W1_slots", 2 * nw), _dev(W2_slots, dt, "W2_slots", nw), _stream()),
        "symi_adam_to_replicas")


def symi_adam_to_replicas_active(cfg, hp, dW1_class, dW2_class, master_w, m, v, slot_offsets,
                                 first_slot, first_slot_next, W1_slots, W2_slots):
    dt = cfg.torch_dtype
    ne = cfg.E * cfg.d * cfg.f
    nw = cfg.S_tot * cfg.d * cfg.f
    per = cfg.E * (3 * cfg.d * cfg.f // cfg.N)
    _check(lib().symi_adam_to_replicas_active(
        ctypes.byref(cfg), ctypes.byref(hp), _dev(dW1_class, F32, "dW1_class", 2 * ne),
        _dev(dW2_class, F32, "dW2_class", ne), _dev(master_w, F32, "master_w", per),
        _dev(m, F32, "m", per), _dev(v, F32, "v", per),
        _dev(slot_offsets, I32, "slot_offsets", cfg.S_tot + 1),
        _dev(first_slot, I32, "first_slot", cfg.E + 1),
        _dev(first_slot_next, I32, "first_slot_next", cfg.E + 1),
        _dev(W1_slots, dt, "W1_slots", 2 * nw), _dev(W2_slots, dt, "W2_slots", nw), _stream()),
        "symi_adam_to_replicas_active")
