"""MI355X-native hot path of Symi's adaptive MoE training step (one GPU's share).

All computation happens in libsymi.so (hand-written HIP for gfx950, C ABI declared in
include/symi.h).  This package only marshals arguments: torch tensors in, pointers out.
"""
from .binding import (  # noqa: F401
    SymiCfg,
    SymiAdam,
    SymiError,
    lib,
    lib_path,
    symi_validate,
    symi_workspace_bytes,
    symi_last_error,
    symi_route,
    symi_route_bwd,
    symi_place,
    symi_place_host,
    symi_dispatch,
    symi_slot_capacity,
    symi_grad_source,
    symi_collect_grads,
    symi_rank_group,
    symi_comm_cost,
    symi_dispatch_capacity,
    symi_dispatch_bwd,
    symi_expert_fwd,
    symi_expert_bwd,
    symi_combine,
    symi_combine_bwd,
    symi_adam_to_replicas,
    symi_timing_enable,
    symi_timing_reset,
    symi_timing_read,
    symi_kernel_count,
    symi_kernel_name,
    EXPORTS,
)
