"""Seeded synthetic workloads for the Symi MoE hot path.

This package only *draws inputs* (token embeddings, router logits, expert weights,
upstream gradients, bias schedules).  It contains none of the method's arithmetic:
no top-k, no placement, no permutation, no FFN, no Adam.  Both the CPU oracle's
tests and the HIP path's tests/bench read their inputs from here so that the two
sides see identical bits.
"""
from .configs import CONFIGS, Config, get_config, scaled  # noqa: F401
from .gen import (  # noqa: F401
    make_logits,
    make_tokens,
    make_class_weights,
    make_upstream_grad,
    bias_schedule,
    make_router,
)
