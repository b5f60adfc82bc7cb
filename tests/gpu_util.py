"""Helpers shared by the GPU parity tests: move synthetic tensors to the device, run the layer
through the C ABI, pick thresholds with a guard band."""
from __future__ import annotations

import numpy as np

from synth import LayerSpec
from threshold_util import pick_tau, spread_thresholds  # noqa: F401  (re-exported for the GPU tests)


def to_dev(a, device="cuda:0"):
    import torch
    if a is None:
        return None
    if a.dtype == np.uint16:  # bf16 bit patterns
        return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(a).to(device)


def to_host64(t, dtype: str) -> np.ndarray:
    import torch
    if dtype == "bf16":
        return t.to(torch.float32).cpu().numpy().astype(np.float64)
    return t.cpu().numpy().astype(np.float64)


def make_gpu_layer(spec: LayerSpec, tensors, max_tokens=None, renorm=False, y_fp32=False, h_scale_log2=0, partial_fp32=False, tall_items=0):
    from paper_2508_18376_amd import DualSparseLayer
    layer = DualSparseLayer(d_model=spec.D, d_ff=spec.F, n_experts=spec.E, top_k=spec.K, n_part=spec.P,
                            max_tokens=max_tokens or max(spec.T, 1), dtype=spec.dtype, n_shared=spec.n_shared,
                            d_ff_shared=spec.F_sh, expert_lo=spec.lo, expert_hi=spec.hi, renorm_combine=renorm,
                            y_fp32=y_fp32, h_scale_log2=h_scale_log2, partial_fp32=partial_fp32, tall_items=tall_items)
    dev = {k: to_dev(v) for k, v in tensors.items() if v is not None}
    layer.partition_weights(dev["w1"], dev["w3"], dev["w2"], perm=dev.get("perm"), sh_w1=dev.get("sh_w1"),
                            sh_w3=dev.get("sh_w3"), sh_w2=dev.get("sh_w2"))
    return layer, dev


def tau_table(spec: LayerSpec, v) -> np.ndarray:
    v = np.asarray(v, dtype=np.float32)
    if v.ndim == 0:
        return np.full((spec.E, spec.P), float(v), dtype=np.float32)
    if v.ndim == 1:
        return np.ascontiguousarray(np.tile(v[None, :], (spec.E, 1)), dtype=np.float32)
    return np.ascontiguousarray(v, dtype=np.float32)


GUARD = 1e-6  # |n - tau| every test input must keep: ~20x the fp32 evaluation error of n (<= 5e-8 for n <= 1)


def rel_err(y_gpu: np.ndarray, y_ref: np.ndarray) -> float:
    rms = float(np.sqrt(np.mean(y_ref ** 2)))
    if rms == 0.0:
        return float(np.abs(y_gpu - y_ref).max())
    return float(np.abs(y_gpu - y_ref).max() / rms)


TOL = {"f32": 1e-5, "bf16": 2e-2}


def bf16_floor(y_ref: np.ndarray) -> float:
    """max |round_bf16(y_ref) - y_ref| / RMS: what rounding the exact result to bf16 costs by itself."""
    from synth import f32_to_bf16_bits, bf16_bits_to_f32
    yb = bf16_bits_to_f32(f32_to_bf16_bits(y_ref.astype(np.float32))).astype(np.float64)
    return rel_err(yb, y_ref)


BF16_HALF_ULP = 2.0 ** -8  # largest relative error of rounding a value to bf16 (8 significant bits)


def assert_output_close(y: np.ndarray, y_ref: np.ndarray, dtype: str, y_fp32: bool = False) -> float:
    """The parity bar for layer outputs.

    fp32 layers: max |err| <= 1e-5 x RMS(y_ref).
    bf16 layers whose output is stored as fp32 (cfg.y_fp32): max |err| <= 2e-2 x RMS(y_ref), the
    plain bar: everything the computation does (bf16 operands, fp32 accumulation, the rounding of
    the intermediate activation) is inside it.
    bf16 layers with a bf16 output: storing the result as bf16 costs up to 2^-8 |y| on any
    implementation (the exact result rounded to bf16 already misses 2e-2 x RMS on outputs whose
    largest element is beyond ~5 RMS), so the elementwise bar is
        |y - y_ref| <= 2e-2 x RMS(y_ref) + 2^-8 |y_ref|,
    and where the rounding floor leaves room (floor <= 1e-2) the plain bar is asserted too.
    Returns max |err| / RMS.
    """
    assert np.isfinite(y).all()
    err = rel_err(y, y_ref)
    if dtype == "f32":
        assert err <= TOL["f32"], (err, TOL["f32"])
        return err
    rms = float(np.sqrt(np.mean(y_ref ** 2)))
    if y_fp32:
        assert err <= TOL["bf16"], (err, TOL["bf16"])
    else:
        excess = np.abs(y - y_ref) - BF16_HALF_ULP * np.abs(y_ref)
        assert excess.max() <= TOL["bf16"] * rms, (excess.max() / max(rms, 1e-300), TOL["bf16"])
        if bf16_floor(y_ref) <= 1e-2:
            assert err <= TOL["bf16"], (err, TOL["bf16"])
    dead = np.abs(y_ref).max(axis=1) == 0
    assert np.all(y[dead] == 0.0)
    return err
