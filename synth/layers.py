"""Layer shapes and seeded random tensors.

Every tensor has its own random stream keyed by (seed, tensor kind, expert index), so a caller
can draw only the router logits of a large layer without paying for its weights, and the values
do not depend on the order in which tensors are drawn.

bf16 tensors are returned as uint16 bit patterns (numpy has no bf16 type); both consumers widen
them themselves.
"""
from __future__ import annotations

import math
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace
from typing import Dict, Optional, Tuple

import numpy as np

_KIND = {"x": 1, "logits": 2, "w1": 3, "w3": 4, "w2": 5, "sh_w1": 6, "sh_w3": 7, "sh_w2": 8, "perm": 9, "wg": 10}


@dataclass(frozen=True)
class LayerSpec:
    name: str
    T: int            # tokens
    D: int            # d_model
    F: int            # d_ff of one routed expert
    E: int            # routed experts (router width)
    K: int            # top-k
    P: int            # partitions per expert
    dtype: str        # "f32" or "bf16": element type of x, weights and y
    seed: int
    n_shared: int = 0     # always-on experts
    F_sh: int = 0         # d_ff of one shared expert
    resident: Optional[Tuple[int, int]] = None  # [lo, hi) routed experts held on this GPU
    x_std: float = 1.0
    w_std: float = 0.02
    zipf_s: float = 0.0   # >0: add a Zipf(s) popularity bias to the router logits
    zipf_rank: Optional[Tuple[int, ...]] = None  # popularity rank (1 = hottest) of each expert id
    perm_kind: str = "random"  # "random" | "identity" | "reversed"

    @property
    def lo(self) -> int:
        return 0 if self.resident is None else self.resident[0]

    @property
    def hi(self) -> int:
        return self.E if self.resident is None else self.resident[1]

    @property
    def E_res(self) -> int:
        return self.hi - self.lo

    def with_(self, **kw) -> "LayerSpec":
        return replace(self, **kw)


# The five benchmark layers.  Shapes stand in for: a unit-test layer, a Mixtral-8x7B layer, a
# fine-grained 64-expert layer, a shared-plus-routed layer, and one expert-parallel rank's share
# of a Mixtral-shaped layer under skewed expert popularity.
LAYERS: Dict[str, LayerSpec] = {
    "C1": LayerSpec("C1", T=64, D=128, F=256, E=8, K=2, P=2, dtype="f32", seed=0, x_std=0.02),
    "C2": LayerSpec("C2", T=4096, D=4096, F=14336, E=8, K=2, P=4, dtype="bf16", seed=1),
    "C3": LayerSpec("C3", T=8192, D=2048, F=1024, E=64, K=8, P=2, dtype="bf16", seed=2),
    "C4": LayerSpec("C4", T=8192, D=2048, F=1408, E=64, K=6, P=2, dtype="bf16", seed=3,
                    n_shared=2, F_sh=1408),
    # expert 0 is the most popular (rank 1), expert 1 has rank 5; both are resident.
    "C5": LayerSpec("C5", T=16384, D=4096, F=14336, E=8, K=2, P=4, dtype="bf16", seed=4,
                    resident=(0, 2), zipf_s=1.2, zipf_rank=(1, 5, 2, 3, 4, 6, 7, 8)),
}


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (round to nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _rng(seed: int, kind: str, sub: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(np.random.SeedSequence([seed, _KIND[kind], sub])))


def _normal(seed: int, kind: str, sub: int, shape, std: float, dtype: str) -> np.ndarray:
    g = _rng(seed, kind, sub)
    a = g.standard_normal(shape, dtype=np.float32)
    a *= np.float32(std)
    return f32_to_bf16_bits(a) if dtype == "bf16" else a


def zipf_logit_bias(spec: LayerSpec) -> np.ndarray:
    """log of the normalised Zipf(s) popularity of each expert id (zeros if zipf_s == 0)."""
    if spec.zipf_s <= 0:
        return np.zeros(spec.E, dtype=np.float32)
    rank = np.asarray(spec.zipf_rank if spec.zipf_rank is not None else range(1, spec.E + 1), dtype=np.float64)
    w = rank ** (-spec.zipf_s)
    return np.log(w / w.sum()).astype(np.float32)


def make_logits(spec: LayerSpec) -> np.ndarray:
    """Router logits [T][E] float32 ~ N(0,1), plus the popularity bias if the layer has one."""
    l = _rng(spec.seed, "logits").standard_normal((spec.T, spec.E), dtype=np.float32)
    if spec.zipf_s > 0:
        l = (l + zipf_logit_bias(spec)[None, :]).astype(np.float32)
    return l


def make_router(spec: LayerSpec) -> np.ndarray:
    """Gating weights W_g [D][E] in the layer's dtype ~ N(0, 1 / (x_std sqrt(D))), so that the logits
    x W_g are ~ N(0, 1) like make_logits' (no popularity bias)."""
    return _normal(spec.seed, "wg", 0, (spec.D, spec.E), 1.0 / (spec.x_std * np.sqrt(spec.D)), spec.dtype)


def make_perm(spec: LayerSpec) -> np.ndarray:
    """perm[e][j] = original neuron placed at new position j, int32 [E_res][F]."""
    out = np.empty((spec.E_res, spec.F), dtype=np.int32)
    for i in range(spec.E_res):
        if spec.perm_kind == "identity":
            out[i] = np.arange(spec.F, dtype=np.int32)
        elif spec.perm_kind == "reversed":
            out[i] = np.arange(spec.F - 1, -1, -1, dtype=np.int32)
        else:
            out[i] = _rng(spec.seed, "perm", spec.lo + i).permutation(spec.F).astype(np.int32)
    return out


def make_layer(spec: LayerSpec, weights: bool = True, threads: int = 8) -> Dict[str, np.ndarray]:
    """All tensors of one layer.

    x [T][D]; logits [T][E] f32; w1, w3 [E_res][D][F]; w2 [E_res][F][D];
    sh_w1, sh_w3 [n_shared][D][F_sh]; sh_w2 [n_shared][F_sh][D]; perm [E_res][F] int32.
    Weight tensors cover only the resident experts (global ids lo..hi-1, in that order).
    """
    t: Dict[str, np.ndarray] = {}
    t["x"] = _normal(spec.seed, "x", 0, (spec.T, spec.D), spec.x_std, spec.dtype)
    t["logits"] = make_logits(spec)
    t["perm"] = make_perm(spec)
    if not weights:
        return t
    el = np.uint16 if spec.dtype == "bf16" else np.float32
    t["w1"] = np.empty((spec.E_res, spec.D, spec.F), dtype=el)
    t["w3"] = np.empty((spec.E_res, spec.D, spec.F), dtype=el)
    t["w2"] = np.empty((spec.E_res, spec.F, spec.D), dtype=el)
    jobs = []
    for i in range(spec.E_res):
        e = spec.lo + i
        jobs.append(("w1", i, e, (spec.D, spec.F)))
        jobs.append(("w3", i, e, (spec.D, spec.F)))
        jobs.append(("w2", i, e, (spec.F, spec.D)))
    if spec.n_shared:
        t["sh_w1"] = np.empty((spec.n_shared, spec.D, spec.F_sh), dtype=el)
        t["sh_w3"] = np.empty((spec.n_shared, spec.D, spec.F_sh), dtype=el)
        t["sh_w2"] = np.empty((spec.n_shared, spec.F_sh, spec.D), dtype=el)
        for s in range(spec.n_shared):
            jobs.append(("sh_w1", s, s, (spec.D, spec.F_sh)))
            jobs.append(("sh_w3", s, s, (spec.D, spec.F_sh)))
            jobs.append(("sh_w2", s, s, (spec.F_sh, spec.D)))

    def run(job):
        kind, slot, sub, shape = job
        t[kind][slot] = _normal(spec.seed, kind, sub, shape, spec.w_std, spec.dtype)

    if threads > 1 and len(jobs) > 1:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(run, jobs))
    else:
        for j in jobs:
            run(j)
    return t


def _selfcheck() -> None:
    a = np.array([1.0, 1.00390625, 1.01171875, -2.5, 0.0], dtype=np.float32)
    b = bf16_bits_to_f32(f32_to_bf16_bits(a))
    assert b[0] == 1.0 and b[3] == -2.5 and b[4] == 0.0
    assert math.isclose(float(b[1]), 1.0)  # tie rounds to even mantissa


if __name__ == "__main__":
    _selfcheck()
    print("ok")
