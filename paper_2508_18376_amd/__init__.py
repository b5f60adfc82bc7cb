"""DualSparse-MoE layer forward on MI355X: thin Python binding over libdsmoe.so.

Every step of the layer runs in the HIP kernels of the shared library; this package only
marshals arguments.  PyTorch is used for device memory and streams.  There is no CPU fallback:
the first use of anything from `binding` without a built library raises.  (`build` and
`thresholds` are plain Python and importable before the library exists.)
"""
import importlib

_BINDING_NAMES = (
    "DsmoeError",
    "DualSparseLayer",
    "dsmoe_create",
    "dsmoe_destroy",
    "dsmoe_packed_bytes",
    "dsmoe_workspace_bytes",
    "dsmoe_strerror",
    "dsmoe_uses_mfma",
    "dsmoe_plan_layout",
    "dsmoe_profile_begin",
    "dsmoe_profile_end",
    "KERNEL_NAMES",
    "moe_partition_weights",
    "moe_route_and_mask",
    "moe_dualsparse_forward",
    "moe_dualsparse_forward_static",
    "dsmoe_static_workspace_need",
    "DSMOE_STATIC_SCRATCH_BYTES",
    "moe_profile_importance",
    "moe_importance_to_perm",
    "moe_select_thresholds",
    "moe_thresholds_for_drop_rate",
    "moe_pack_router",
    "moe_router_logits",
    "moe_dualsparse_forward_routed",
    "moe_transform_complete",
    "dsmoe_router_packed_bytes",
    "lib_path",
)
__all__ = list(_BINDING_NAMES)


def __getattr__(name):
    # the binding loads libdsmoe.so when it is imported; defer that to the first use so that the
    # build script, which lives in this package, can run on a tree that has no library yet
    if name in _BINDING_NAMES or name == "binding":
        mod = importlib.import_module(".binding", __name__)
        return mod if name == "binding" else getattr(mod, name)
    raise AttributeError("module %r has no attribute %r" % (__name__, name))
