"""Rectify-Router MoE-layer forward (and the router-score gradient of its weights) for AMD MI355X (gfx950).

The product is the HIP library `librr.so` (C ABI in include/rr.h); `binding` marshals torch
tensors into it and `workloads` draws seeded synthetic inputs.  There is no CPU fallback: every
call raises if the library is missing.
"""
from .binding import (  # noqa: F401
    RRConfig, RRError, Tables, alloc_tables, alloc_workspace, library_path, load_library,
    rr_capacity, rr_init, rr_moe_forward, rr_profile_enable, rr_profile_read, rr_rectified_dispatch,
    rr_rectified_dispatch_static,
    rr_router_backward, rr_router_scores, rr_slots_per_expert, rr_strerror, rr_workspace_bytes,
    RR_F32, RR_BF16, RR_ACT_GELU, RR_ACT_SWIGLU, RR_INTRA_GPU, RR_FILL_IN, RR_POLICY_ARRIVAL,
    RR_QUOTA_PER_GROUP, RR_GRAD_STRAIGHT_THROUGH,
)
