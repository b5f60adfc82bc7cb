"""DualSparse-MoE layer forward on MI355X: thin Python binding over libdsmoe.so.

Every step of the layer runs in the HIP kernels of the shared library; this package only
marshals arguments.  PyTorch is used for device memory and streams.  There is no CPU fallback:
importing `binding` without a built library raises.
"""
from .binding import (  # noqa: F401
    DsmoeError,
    DualSparseLayer,
    dsmoe_create,
    dsmoe_destroy,
    dsmoe_packed_bytes,
    dsmoe_workspace_bytes,
    dsmoe_strerror,
    dsmoe_uses_mfma,
    dsmoe_plan_layout,
    dsmoe_profile_begin,
    dsmoe_profile_end,
    KERNEL_NAMES,
    moe_partition_weights,
    moe_route_and_mask,
    moe_dualsparse_forward,
    moe_profile_importance,
    moe_importance_to_perm,
    moe_select_thresholds,
    moe_thresholds_for_drop_rate,
    moe_pack_router,
    moe_router_logits,
    moe_dualsparse_forward_routed,
    moe_transform_complete,
    dsmoe_router_packed_bytes,
    lib_path,
)
