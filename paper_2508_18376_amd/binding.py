"""ctypes marshalling for include/dsmoe.h.  Same names as the C ABI; tensors are torch tensors on
the GPU, passed as raw device pointers."""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libdsmoe.so")  # the in-tree build, nothing else

DSMOE_F32, DSMOE_BF16 = 0, 1
DSMOE_PLAN_FIELDS = 14


class DsmoeError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %d (%s)" % (where, status, dsmoe_strerror(status)))


class _Config(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "d_model", "d_ff", "n_experts", "top_k", "n_part", "n_shared", "d_ff_shared", "expert_lo", "expert_hi",
        "renorm_combine", "max_tokens", "dtype", "y_fp32", "h_scale_log2", "partial_fp32", "tall_items")]


def lib_path() -> str:
    return _LIB_PATH


def _load() -> ctypes.CDLL:
    if not os.path.exists(_LIB_PATH):
        raise ImportError("libdsmoe.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(there is no fallback path)")
    L = ctypes.CDLL(_LIB_PATH)
    vp, i32, i64p = ctypes.c_void_p, ctypes.c_int32, ctypes.POINTER(ctypes.c_int64)
    L.dsmoe_create.argtypes = [ctypes.POINTER(_Config), ctypes.POINTER(vp)]
    L.dsmoe_create.restype = ctypes.c_int
    L.dsmoe_destroy.argtypes = [vp]
    L.dsmoe_destroy.restype = ctypes.c_int
    L.dsmoe_packed_bytes.argtypes = [vp]
    L.dsmoe_packed_bytes.restype = ctypes.c_size_t
    L.dsmoe_workspace_bytes.argtypes = [vp]
    L.dsmoe_workspace_bytes.restype = ctypes.c_size_t
    L.dsmoe_strerror.argtypes = [ctypes.c_int]
    L.dsmoe_strerror.restype = ctypes.c_char_p
    L.dsmoe_last_hip_error.argtypes = [vp]
    L.dsmoe_last_hip_error.restype = ctypes.c_int
    L.dsmoe_uses_mfma.argtypes = [vp]
    L.dsmoe_uses_mfma.restype = ctypes.c_int
    L.moe_partition_weights.argtypes = [vp] * 10
    L.moe_partition_weights.restype = ctypes.c_int
    L.moe_route_and_mask.argtypes = [vp, vp, i32, vp, vp, vp, vp, vp, vp]
    L.moe_route_and_mask.restype = ctypes.c_int
    L.moe_dualsparse_forward.argtypes = [vp, vp, vp, vp, vp, i32, vp, vp, vp]
    L.moe_dualsparse_forward.restype = ctypes.c_int
    L.moe_dualsparse_forward_static.argtypes = [vp, vp, vp, vp, vp, i32, vp, vp]
    L.moe_dualsparse_forward_static.restype = ctypes.c_int
    L.dsmoe_static_workspace_need.argtypes = [vp, i32]
    L.dsmoe_static_workspace_need.restype = ctypes.c_size_t
    L.moe_profile_importance.argtypes = [vp, vp, vp, vp, i32, i32, vp, vp, vp]
    L.moe_profile_importance.restype = ctypes.c_int
    L.moe_importance_to_perm.argtypes = [vp, vp, vp, vp]
    L.moe_importance_to_perm.restype = ctypes.c_int
    L.dsmoe_router_packed_bytes.argtypes = [vp]
    L.dsmoe_router_packed_bytes.restype = ctypes.c_size_t
    L.moe_pack_router.argtypes = [vp, vp, vp, vp]
    L.moe_pack_router.restype = ctypes.c_int
    L.moe_router_logits.argtypes = [vp, vp, vp, i32, vp, vp]
    L.moe_router_logits.restype = ctypes.c_int
    L.moe_dualsparse_forward_routed.argtypes = [vp, vp, vp, vp, vp, i32, vp, vp, vp, vp]
    L.moe_dualsparse_forward_routed.restype = ctypes.c_int
    L.moe_transform_complete.argtypes = [vp] * 12
    L.moe_transform_complete.restype = ctypes.c_int
    L.moe_thresholds_for_drop_rate.argtypes = [vp, vp, i32, ctypes.c_double, ctypes.POINTER(ctypes.c_int32), vp, vp, vp, vp]
    L.moe_thresholds_for_drop_rate.restype = ctypes.c_int
    L.moe_select_thresholds.argtypes = [vp, vp, i32, vp, i32, i32, vp, vp, vp, vp]
    L.moe_select_thresholds.restype = ctypes.c_int
    L.dsmoe_plan_layout.argtypes = [vp, i64p]
    L.dsmoe_plan_layout.restype = ctypes.c_int
    L.dsmoe_profile_begin.argtypes = [vp, ctypes.c_int, ctypes.c_int]
    L.dsmoe_profile_begin.restype = ctypes.c_int
    L.dsmoe_profile_end.argtypes = [vp, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_int)]
    L.dsmoe_profile_end.restype = ctypes.c_int
    return L


_lib = _load()


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "tensors must be contiguous GPU tensors"
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def dsmoe_strerror(status: int) -> str:
    return _lib.dsmoe_strerror(int(status)).decode()


def dsmoe_create(*, d_model, d_ff, n_experts, top_k, n_part, max_tokens, dtype, n_shared=0, d_ff_shared=0,
                 expert_lo=0, expert_hi=None, renorm_combine=0, y_fp32=0, h_scale_log2=0,
                 partial_fp32=0, tall_items=0) -> ctypes.c_void_p:
    cfg = _Config(d_model, d_ff, n_experts, top_k, n_part, n_shared, d_ff_shared, expert_lo,
                  n_experts if expert_hi is None else expert_hi, int(renorm_combine), max_tokens, dtype, int(y_fp32),
                  int(h_scale_log2), int(partial_fp32), int(tall_items))
    out = ctypes.c_void_p()
    rc = _lib.dsmoe_create(ctypes.byref(cfg), ctypes.byref(out))
    if rc != 0:
        raise DsmoeError(rc, "dsmoe_create")
    return out


def dsmoe_destroy(ctx) -> None:
    _lib.dsmoe_destroy(ctx)


def dsmoe_packed_bytes(ctx) -> int:
    return int(_lib.dsmoe_packed_bytes(ctx))


def dsmoe_workspace_bytes(ctx) -> int:
    return int(_lib.dsmoe_workspace_bytes(ctx))


def dsmoe_uses_mfma(ctx) -> bool:
    return bool(_lib.dsmoe_uses_mfma(ctx))


def dsmoe_plan_layout(ctx):
    out = (ctypes.c_int64 * DSMOE_PLAN_FIELDS)()
    n = _lib.dsmoe_plan_layout(ctx, out)
    if n < 0:
        raise DsmoeError(n, "dsmoe_plan_layout")
    return [int(v) for v in out]


KERNEL_NAMES = ("router", "route_mask", "plan", "scatter", "gemm1", "gemm2", "combine")


def dsmoe_profile_begin(ctx, level: int, max_calls: int) -> None:
    _check(_lib.dsmoe_profile_begin(ctx, int(level), int(max_calls)), ctx, "dsmoe_profile_begin")


def dsmoe_profile_end(ctx):
    """Returns ({kernel name: mean ms}, recorded calls)."""
    ms = (ctypes.c_float * len(KERNEL_NAMES))()
    calls = ctypes.c_int(0)
    _check(_lib.dsmoe_profile_end(ctx, ms, ctypes.byref(calls)), ctx, "dsmoe_profile_end")
    return {k: float(ms[i]) for i, k in enumerate(KERNEL_NAMES)}, int(calls.value)


def _check(rc: int, ctx, where: str) -> None:
    if rc != 0:
        e = DsmoeError(rc, where)
        if rc == -4:
            e.args = (e.args[0] + " hipError=%d" % _lib.dsmoe_last_hip_error(ctx),)
        raise e


def moe_partition_weights(ctx, w1, w3, w2, sh_w1, sh_w3, sh_w2, perm, packed_out, stream=None) -> None:
    rc = _lib.moe_partition_weights(ctx, _ptr(w1), _ptr(w3), _ptr(w2), _ptr(sh_w1), _ptr(sh_w3), _ptr(sh_w2), _ptr(perm),
                                    _ptr(packed_out), _stream(stream))
    _check(rc, ctx, "moe_partition_weights")


def moe_route_and_mask(ctx, logits, T, tau, topk_idx, topk_w, keep_bits, group_count, stream=None) -> None:
    rc = _lib.moe_route_and_mask(ctx, _ptr(logits), int(T), _ptr(tau), _ptr(topk_idx), _ptr(topk_w), _ptr(keep_bits),
                                 _ptr(group_count), _stream(stream))
    _check(rc, ctx, "moe_route_and_mask")


def moe_dualsparse_forward(ctx, packed, x, logits, tau, T, y, workspace, stream=None) -> None:
    rc = _lib.moe_dualsparse_forward(ctx, _ptr(packed), _ptr(x), _ptr(logits), _ptr(tau), int(T), _ptr(y), _ptr(workspace),
                                     _stream(stream))
    _check(rc, ctx, "moe_dualsparse_forward")


def moe_dualsparse_forward_static(ctx, packed, x, logits, tau, T, y, stream=None) -> None:
    rc = _lib.moe_dualsparse_forward_static(ctx, _ptr(packed), _ptr(x), _ptr(logits), _ptr(tau), int(T), _ptr(y), _stream(stream))
    _check(rc, ctx, "moe_dualsparse_forward_static")


def dsmoe_static_workspace_need(ctx, T) -> int:
    return int(_lib.dsmoe_static_workspace_need(ctx, int(T)))


DSMOE_STATIC_SCRATCH_BYTES = 256 << 20


def moe_profile_importance(ctx, packed, x, logits, T, metric, importance, workspace, stream=None) -> None:
    rc = _lib.moe_profile_importance(ctx, _ptr(packed), _ptr(x), _ptr(logits), int(T), int(metric), _ptr(importance),
                                     _ptr(workspace), _stream(stream))
    _check(rc, ctx, "moe_profile_importance")


def moe_importance_to_perm(ctx, importance, perm, stream=None) -> None:
    _check(_lib.moe_importance_to_perm(ctx, _ptr(importance), _ptr(perm), _stream(stream)), ctx, "moe_importance_to_perm")


def dsmoe_router_packed_bytes(ctx) -> int:
    return int(_lib.dsmoe_router_packed_bytes(ctx))


def moe_pack_router(ctx, wg, router_packed, stream=None) -> None:
    _check(_lib.moe_pack_router(ctx, _ptr(wg), _ptr(router_packed), _stream(stream)), ctx, "moe_pack_router")


def moe_router_logits(ctx, router_packed, x, T, logits, stream=None) -> None:
    _check(_lib.moe_router_logits(ctx, _ptr(router_packed), _ptr(x), int(T), _ptr(logits), _stream(stream)), ctx,
           "moe_router_logits")


def moe_dualsparse_forward_routed(ctx, packed, router_packed, x, tau, T, y, logits_out, workspace, stream=None) -> None:
    rc = _lib.moe_dualsparse_forward_routed(ctx, _ptr(packed), _ptr(router_packed), _ptr(x), _ptr(tau), int(T), _ptr(y),
                                            _ptr(logits_out), _ptr(workspace), _stream(stream))
    _check(rc, ctx, "moe_dualsparse_forward_routed")


def moe_transform_complete(ctx, wg, w1, w3, w2, perm, wg_out, w1_out, w3_out, w2_out, workspace, stream=None) -> None:
    rc = _lib.moe_transform_complete(ctx, _ptr(wg), _ptr(w1), _ptr(w3), _ptr(w2), _ptr(perm), _ptr(wg_out), _ptr(w1_out),
                                     _ptr(w3_out), _ptr(w2_out), _ptr(workspace), _stream(stream))
    _check(rc, ctx, "moe_transform_complete")


def moe_thresholds_for_drop_rate(ctx, logits, T, rate, offset_bins, tau, stats, workspace, stream=None) -> None:
    off = (ctypes.c_int32 * len(offset_bins))(*[int(v) for v in offset_bins])
    rc = _lib.moe_thresholds_for_drop_rate(ctx, _ptr(logits), int(T), ctypes.c_double(rate), off, _ptr(tau), _ptr(stats),
                                           _ptr(workspace), _stream(stream))
    _check(rc, ctx, "moe_thresholds_for_drop_rate")


def moe_select_thresholds(ctx, logits, T, tau_max, group_size, row_cap, tau, pair_count, workspace, stream=None) -> None:
    rc = _lib.moe_select_thresholds(ctx, _ptr(logits), int(T), _ptr(tau_max), int(group_size), int(row_cap), _ptr(tau),
                                    _ptr(pair_count), _ptr(workspace), _stream(stream))
    _check(rc, ctx, "moe_select_thresholds")


class DualSparseLayer:
    """Owns a context plus its packed-weight and workspace buffers (torch allocations)."""

    def __init__(self, *, d_model, d_ff, n_experts, top_k, n_part, max_tokens, dtype="bf16", n_shared=0, d_ff_shared=0,
                 expert_lo=0, expert_hi=None, renorm_combine=False, y_fp32=False, h_scale_log2=0,
                 partial_fp32=False, tall_items=0, device="cuda:0"):
        self.device = torch.device(device)
        self.dtype = dtype
        self.D, self.F, self.E, self.K, self.P = d_model, d_ff, n_experts, top_k, n_part
        self.lo, self.hi = expert_lo, (n_experts if expert_hi is None else expert_hi)
        self.n_shared, self.F_sh = n_shared, d_ff_shared
        self.max_tokens = max_tokens
        self.ctx = dsmoe_create(d_model=d_model, d_ff=d_ff, n_experts=n_experts, top_k=top_k, n_part=n_part,
                                max_tokens=max_tokens, dtype=DSMOE_BF16 if dtype == "bf16" else DSMOE_F32,
                                n_shared=n_shared, d_ff_shared=d_ff_shared, expert_lo=expert_lo, expert_hi=self.hi,
                                renorm_combine=int(bool(renorm_combine)), y_fp32=int(bool(y_fp32)),
                                h_scale_log2=h_scale_log2, partial_fp32=int(bool(partial_fp32)), tall_items=int(tall_items))
        self.packed = torch.empty(dsmoe_packed_bytes(self.ctx), dtype=torch.uint8, device=self.device)
        self.workspace = torch.empty(dsmoe_workspace_bytes(self.ctx), dtype=torch.uint8, device=self.device)
        self.torch_dtype = torch.bfloat16 if dtype == "bf16" else torch.float32  # of x and the weights
        self.y_dtype = torch.float32 if (y_fp32 or dtype != "bf16") else torch.bfloat16

    @property
    def uses_mfma(self) -> bool:
        return dsmoe_uses_mfma(self.ctx)

    def partition_weights(self, w1, w3, w2, perm=None, sh_w1=None, sh_w3=None, sh_w2=None) -> None:
        with torch.cuda.device(self.device):
            moe_partition_weights(self.ctx, w1, w3, w2, sh_w1, sh_w3, sh_w2, perm, self.packed)

    def route_and_mask(self, logits, tau):
        T = logits.shape[0]
        n = max(T * self.K, 1)
        idx = torch.empty(n, dtype=torch.int32, device=self.device)
        w = torch.empty(n, dtype=torch.float32, device=self.device)
        keep = torch.empty(n, dtype=torch.uint8, device=self.device)
        gc = torch.empty(self.E * self.P, dtype=torch.int32, device=self.device)
        with torch.cuda.device(self.device):
            moe_route_and_mask(self.ctx, logits, T, tau, idx, w, keep, gc)
        return idx[:T * self.K].view(T, self.K), w[:T * self.K].view(T, self.K), keep[:T * self.K].view(T, self.K), gc

    def forward(self, x, logits, tau, out=None):
        T = x.shape[0]
        y = out if out is not None else torch.empty((T, self.D), dtype=self.y_dtype, device=self.device)
        assert y.dtype == self.y_dtype
        with torch.cuda.device(self.device):
            moe_dualsparse_forward(self.ctx, self.packed, x, logits, tau, T, y, self.workspace)
        return y

    def profile_importance(self, x, logits, metric):
        """Importance [E_res][F] of the calibration tokens x (weights must be packed with perm=None)."""
        imp = torch.empty((self.hi - self.lo, self.F), dtype=torch.float32, device=self.device)
        with torch.cuda.device(self.device):
            moe_profile_importance(self.ctx, self.packed, x, logits, x.shape[0], metric, imp, self.workspace)
        return imp

    def importance_to_perm(self, importance):
        perm = torch.empty((self.hi - self.lo, self.F), dtype=torch.int32, device=self.device)
        with torch.cuda.device(self.device):
            moe_importance_to_perm(self.ctx, importance, perm)
        return perm

    def pack_router(self, wg):
        """Keeps W_g [D][E] in the kernel's operand order for router_logits / forward_routed."""
        self.router_packed = torch.empty(max(dsmoe_router_packed_bytes(self.ctx), 16), dtype=torch.uint8, device=self.device)
        with torch.cuda.device(self.device):
            moe_pack_router(self.ctx, wg, self.router_packed)

    def router_logits(self, x):
        logits = torch.empty((x.shape[0], self.E), dtype=torch.float32, device=self.device)
        with torch.cuda.device(self.device):
            moe_router_logits(self.ctx, self.router_packed, x, x.shape[0], logits)
        return logits

    def forward_routed(self, x, tau, want_logits=False):
        T = x.shape[0]
        y = torch.empty((T, self.D), dtype=self.y_dtype, device=self.device)
        logits = torch.empty((T, self.E), dtype=torch.float32, device=self.device) if want_logits else None
        with torch.cuda.device(self.device):
            moe_dualsparse_forward_routed(self.ctx, self.packed, self.router_packed, x, tau, T, y, logits, self.workspace)
        return (y, logits) if want_logits else y

    def transform_complete(self, wg, w1, w3, w2, perm=None):
        """(wg', w1', w3', w2') of the equivalent layer with E*P experts (Sec. 3.1)."""
        E_res, P, Fp = self.hi - self.lo, self.P, self.F // self.P
        wg_o = torch.empty((self.D, self.E * P), dtype=wg.dtype, device=self.device) if wg is not None else None
        w1_o = torch.empty((E_res * P, self.D, Fp), dtype=w1.dtype, device=self.device)
        w3_o = torch.empty((E_res * P, self.D, Fp), dtype=w3.dtype, device=self.device)
        w2_o = torch.empty((E_res * P, Fp, self.D), dtype=w2.dtype, device=self.device)
        with torch.cuda.device(self.device):
            moe_transform_complete(self.ctx, wg, w1, w3, w2, perm, wg_o, w1_o, w3_o, w2_o, self.workspace)
        return wg_o, w1_o, w3_o, w2_o

    def thresholds_for_drop_rate(self, logits, rate, offset_bins=None):
        """tau [E][P] that drops at least `rate` of this batch's resident units, and (dropped, total) units."""
        if offset_bins is None:  # the policy's default: -0.01 .. +0.01 around the centre (Sec. 4.2 c)
            from .thresholds import offset_bins as default_offset_bins
            offset_bins = default_offset_bins(self.P)
        assert len(offset_bins) == self.P
        tau = torch.empty((self.E, self.P), dtype=torch.float32, device=self.device)
        stats = torch.empty((2,), dtype=torch.int32, device=self.device)
        with torch.cuda.device(self.device):
            moe_thresholds_for_drop_rate(self.ctx, logits, logits.shape[0], rate, offset_bins, tau, stats, self.workspace)
        return tau, stats

    def select_thresholds(self, logits, tau_max, group_size=1, row_cap=0):
        """Load-aware tau [E][P] (and the pair count of every expert) for this batch, on the device."""
        tau = torch.empty((self.E, self.P), dtype=torch.float32, device=self.device)
        pairs = torch.empty((self.E,), dtype=torch.int32, device=self.device)
        with torch.cuda.device(self.device):
            moe_select_thresholds(self.ctx, logits, logits.shape[0], tau_max, group_size, row_cap, tau, pairs, self.workspace)
        return tau, pairs

    def plan(self, T):
        """Copies of the last forward call's plan arrays (for tests)."""
        lay = dsmoe_plan_layout(self.ctx)
        ws = self.workspace
        n = T * self.K
        rows = lay[8]

        def view(off, count, dt):
            nbytes = count * torch.empty(0, dtype=dt).element_size()
            return ws[off:off + nbytes].view(dt).clone()

        E_res = self.hi - self.lo
        return {
            "topk_idx": view(lay[0], n, torch.int32).view(T, self.K),
            "topk_w": view(lay[1], n, torch.float32).view(T, self.K),
            "keep_bits": view(lay[2], n, torch.uint8).view(T, self.K),
            "pair_row": view(lay[3], n, torch.int32).view(T, self.K),
            "row_token": view(lay[4], rows, torch.int32),
            "row_bits": view(lay[5], rows, torch.uint8),
            "expert_nrows": view(lay[6], E_res, torch.int32),
            "expert_row0": view(lay[7], E_res, torch.int32),
            "row_cap": rows,
            "tile_rows": lay[9],
            "shared_rows": lay[10],
            "counters": view(lay[11], 5, torch.int32),
            "items1": view(lay[12], 8 * int(view(lay[11], 1, torch.int32)[0]), torch.int32).view(-1, 8),
            "items2": view(lay[13], 8 * int(view(lay[11], 2, torch.int32)[1]), torch.int32).view(-1, 8),
        }

    def close(self) -> None:
        if self.ctx is not None:
            dsmoe_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
