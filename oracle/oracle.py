"""ctypes wrapper around dsmoe_oracle.c (compiled with gcc on first use or by build())."""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dsmoe_oracle.c")
_LIB = os.path.join(_HERE, "libdsmoe_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc -O2 -fopenmp.  Returns the path of the shared object."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        L.dsmoe_oracle_threads.restype = ctypes.c_int
        L.dsmoe_oracle_route.restype = ctypes.c_int
        L.dsmoe_oracle_forward.restype = ctypes.c_int
        _lib = L
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def n_threads() -> int:
    return int(_load().dsmoe_oracle_threads())


@dataclass
class RouteResult:
    idx: np.ndarray          # [T][K] int32 expert ids, selection order
    s: np.ndarray            # [T][K] softmax scores
    n: np.ndarray            # [T][K] scores normalised over the K selected
    g: np.ndarray            # [T][K] combine weights (s, or n with renorm)
    keep: np.ndarray         # [T][K][P] uint8
    group_count: np.ndarray  # [E*P] int64 kept units of sub-expert e*P+p
    min_margin: float        # min |n - tau| over resident units

    @property
    def keep_bits(self) -> np.ndarray:
        """[T][K] uint8, bit p set iff partition p is kept."""
        P = self.keep.shape[2]
        w = (1 << np.arange(P)).astype(np.uint32)
        return (self.keep.astype(np.uint32) * w).sum(axis=2).astype(np.uint8)


def route(logits: np.ndarray, K: int, P: int, tau: np.ndarray, lo: int = 0, hi: Optional[int] = None,
          renorm: bool = False) -> RouteResult:
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    T, E = logits.shape
    hi = E if hi is None else hi
    tau = np.ascontiguousarray(tau, dtype=np.float32)
    assert tau.shape == (E, P), (tau.shape, (E, P))
    idx = np.empty((T, K), dtype=np.int32)
    s = np.empty((T, K), dtype=np.float64)
    n = np.empty((T, K), dtype=np.float64)
    g = np.empty((T, K), dtype=np.float64)
    keep = np.empty((T, K, P), dtype=np.uint8)
    gc = np.empty((E * P,), dtype=np.int64)
    mm = ctypes.c_double(0.0)
    rc = _load().dsmoe_oracle_route(_p(logits), T, E, K, P, _p(tau), lo, hi, int(bool(renorm)), _p(idx), _p(s), _p(n),
                                    _p(g), _p(keep), _p(gc), ctypes.byref(mm))
    if rc != 0:
        raise ValueError("dsmoe_oracle_route: bad argument")
    return RouteResult(idx, s, n, g, keep, gc, float(mm.value))


def forward(x: np.ndarray, logits: np.ndarray, w1: np.ndarray, w3: np.ndarray, w2: np.ndarray, tau: np.ndarray, K: int,
            P: int, perm: Optional[np.ndarray] = None, sh_w1: Optional[np.ndarray] = None,
            sh_w3: Optional[np.ndarray] = None, sh_w2: Optional[np.ndarray] = None, lo: int = 0,
            hi: Optional[int] = None, renorm: bool = False, tokens: Optional[np.ndarray] = None) -> np.ndarray:
    """Layer output, float64 [n_tokens][D].  x / weights: float32 arrays, or uint16 arrays of bf16 bits."""
    dtype = 1 if x.dtype == np.uint16 else 0
    el = np.uint16 if dtype else np.float32
    x = np.ascontiguousarray(x, dtype=el)
    w1 = np.ascontiguousarray(w1, dtype=el)
    w3 = np.ascontiguousarray(w3, dtype=el)
    w2 = np.ascontiguousarray(w2, dtype=el)
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    T, D = x.shape
    E = logits.shape[1]
    hi = E if hi is None else hi
    E_res, D2, F = w1.shape
    assert D2 == D and E_res == hi - lo and w3.shape == w1.shape and w2.shape == (E_res, F, D)
    assert logits.shape[0] == T
    tau = np.ascontiguousarray(tau, dtype=np.float32)
    assert tau.shape == (E, P)
    if perm is not None:
        perm = np.ascontiguousarray(perm, dtype=np.int32)
        assert perm.shape == (E_res, F)
    n_shared, F_sh = 0, 0
    if sh_w1 is not None:
        sh_w1 = np.ascontiguousarray(sh_w1, dtype=el)
        sh_w3 = np.ascontiguousarray(sh_w3, dtype=el)
        sh_w2 = np.ascontiguousarray(sh_w2, dtype=el)
        n_shared, _, F_sh = sh_w1.shape
        assert sh_w1.shape == (n_shared, D, F_sh) and sh_w3.shape == sh_w1.shape and sh_w2.shape == (n_shared, F_sh, D)
    if tokens is None:
        n_tok = T
    else:
        tokens = np.ascontiguousarray(tokens, dtype=np.int32)
        n_tok = int(tokens.shape[0])
    y = np.empty((n_tok, D), dtype=np.float64)
    rc = _load().dsmoe_oracle_forward(_p(x), _p(logits), _p(w1), _p(w3), _p(w2), _p(sh_w1), _p(sh_w3), _p(sh_w2),
                                      _p(perm), _p(tau), T, D, F, E, K, P, n_shared, F_sh, lo, hi, int(bool(renorm)),
                                      dtype, _p(tokens), n_tok, _p(y))
    if rc != 0:
        raise ValueError("dsmoe_oracle_forward: bad argument")
    return y


def importance(x: np.ndarray, logits: np.ndarray, w1: np.ndarray, w3: np.ndarray, K: int, metric: int, lo: int = 0,
               hi: Optional[int] = None):
    """Accumulated neuron importance [E_res][F] (float64) and the sum of the terms' absolute values."""
    dtype = 1 if x.dtype == np.uint16 else 0
    el = np.uint16 if dtype else np.float32
    x = np.ascontiguousarray(x, dtype=el)
    w1 = np.ascontiguousarray(w1, dtype=el)
    w3 = np.ascontiguousarray(w3, dtype=el)
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    T, D = x.shape
    E = logits.shape[1]
    hi = E if hi is None else hi
    E_res, _, F = w1.shape
    assert E_res == hi - lo and w3.shape == w1.shape and logits.shape[0] == T
    L = _load()
    L.dsmoe_oracle_importance.restype = ctypes.c_int
    imp = np.empty((E_res, F), dtype=np.float64)
    ab = np.empty((E_res, F), dtype=np.float64)
    rc = L.dsmoe_oracle_importance(_p(x), _p(logits), _p(w1), _p(w3), T, D, F, E, K, lo, hi, dtype, int(metric), _p(imp), _p(ab))
    if rc != 0:
        raise ValueError("dsmoe_oracle_importance: bad argument")
    return imp, ab


def perm_from_importance(imp: np.ndarray) -> np.ndarray:
    """perm[e][j] = neuron with the j-th largest importance, ties to the lower neuron id (Sec. 4.2 b)."""
    out = np.empty(imp.shape, dtype=np.int32)
    for e in range(imp.shape[0]):
        out[e] = np.lexsort((np.arange(imp.shape[1]), -imp[e])).astype(np.int32)
    return out


@dataclass
class ThresholdSelection:
    tau: np.ndarray          # [E][P] float32
    pair_count: np.ndarray   # [E] int64 Top-K pairs per expert, nothing dropped
    ratio: np.ndarray        # [E/group_size] float32 actual / ideal load of each device
    cap_bin: np.ndarray      # [E] int64 grid index b of the row-cap threshold b / n_bins (0 = cap not binding)
    min_margin: float        # min distance of a score to the two grid values that decide cap_bin


def select_thresholds(logits: np.ndarray, K: int, P: int, tau_max: np.ndarray, group_size: int = 1, row_cap: int = 0,
                      n_bins: int = 4096) -> ThresholdSelection:
    """Load-aware thresholds (Sec. 4.3) and the score-distribution map from a row budget to a
    threshold (Sec. 5.3.3 observes that the threshold <-> drop-rate relation is not linear).

    Device d holds experts [d*group_size, (d+1)*group_size).  Its load ratio is r = pairs routed
    to its experts / (T*K*group_size/E).  r >= 1: its experts take tau_max; r < 1: tau_max * r.
    With row_cap > 0 every expert's thresholds are then lifted, keeping their spacing, until at
    most row_cap of its pairs reach the lowest of them; the lifted minimum is the smallest value
    b / n_bins (b integer) that achieves this.  All threshold arithmetic is single precision, the
    precision in which the thresholds are compared with the scores."""
    f32 = np.float32
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    T, E = logits.shape
    tau_max = np.asarray(tau_max, dtype=np.float32)
    assert tau_max.shape == (P,) and E % group_size == 0
    r = route(logits, K, P, np.zeros((E, P), np.float32))
    n = r.n.astype(np.float32)
    pair_count = np.array([(r.idx == e).sum() for e in range(E)], dtype=np.int64)
    n_dev = E // group_size
    ideal = f32(T * K * group_size) / f32(E)
    ratio = np.empty(n_dev, dtype=np.float32)
    tau = np.empty((E, P), dtype=np.float32)
    cap_bin = np.zeros(E, dtype=np.int64)
    margin = np.inf
    for d in range(n_dev):
        load = int(pair_count[d * group_size:(d + 1) * group_size].sum())
        ratio[d] = f32(load) / ideal
        scale = ratio[d] if ratio[d] < f32(1) else f32(1)
        for e in range(d * group_size, (d + 1) * group_size):
            tau[e] = tau_max * scale
    if row_cap > 0:
        for e in range(E):
            ne = n[r.idx == e]
            b = 0
            while int((ne >= f32(b) / f32(n_bins)).sum()) > row_cap:  # ends at the latest at b = n_bins + 1 (> any score)
                b += 1
            cap_bin[e] = b
            floor_e = f32(b) / f32(n_bins)
            lowest = tau[e].min()
            if floor_e > lowest:
                tau[e] = floor_e + (tau[e] - lowest)
            if b > 0 and ne.size:
                for edge in (b, b - 1):
                    margin = min(margin, float(np.abs(ne.astype(np.float64) - edge / n_bins).min()))
    return ThresholdSelection(tau, pair_count, ratio, cap_bin, float(margin))


def _widen(a: np.ndarray) -> np.ndarray:
    """float64 view of an input tensor: float32 as is, uint16 as bfloat16 bit patterns (exact)."""
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def _narrow_like(v: np.ndarray, like: np.ndarray) -> np.ndarray:
    """Round float64 values to the storage type of `like` (float32, or bfloat16 bits, nearest-even)."""
    f = v.astype(np.float32)
    if like.dtype != np.uint16:
        return f
    b = f.view(np.uint32)
    return ((b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)).astype(np.uint16)


def router_logits(x: np.ndarray, wg: np.ndarray) -> np.ndarray:
    """Gating logits l = x W_g (Sec. 3.1, first equation; W_g is [d_model][E]), float64 [T][E]."""
    return np.matmul(_widen(x), _widen(wg))


def complete_transform(wg: np.ndarray, w1: np.ndarray, w3: np.ndarray, w2: np.ndarray, P: int,
                       perm: Optional[np.ndarray] = None, scale_w2: bool = True):
    """Complete transformation of a layer into E*P finer-grained experts (Sec. 3.1, steps 1-3).

    Router column e is repeated P times (new experts e*P .. e*P+P-1); the neurons of expert e, in
    the order perm[e] (Sec. 4.2 b; identity if None), are split evenly so that new expert e*P+p
    owns positions [p*F/P, (p+1)*F/P); its down projection is multiplied by P (rounded once to the
    storage type).  Returns (wg', w1', w3', w2') with shapes [D][E*P], [E*P][D][F/P] (twice),
    [E*P][F/P][D]; the transformed layer selects Top-(K*P)."""
    E, D, F = w1.shape
    assert F % P == 0 and wg.shape == (D, E)
    Fp = F // P
    wg_t = np.repeat(wg, P, axis=1)
    w1_t = np.empty((E * P, D, Fp), dtype=w1.dtype)
    w3_t = np.empty((E * P, D, Fp), dtype=w3.dtype)
    w2_t = np.empty((E * P, Fp, D), dtype=w2.dtype)
    for e in range(E):
        order = np.arange(F) if perm is None else perm[e]
        for p in range(P):
            own = order[p * Fp:(p + 1) * Fp]
            w1_t[e * P + p] = w1[e][:, own]
            w3_t[e * P + p] = w3[e][:, own]
            rows = w2[e][own, :]
            w2_t[e * P + p] = _narrow_like(_widen(rows) * P, w2) if scale_w2 else rows
    return wg_t, w1_t, w3_t, w2_t


@dataclass
class DropRateThresholds:
    tau: np.ndarray        # [E][P] float32, the same row for every expert
    centre_bin: int        # b: thresholds are (b + offset_bins[p]) / n_bins
    dropped_units: int     # units of resident pairs below their threshold
    total_units: int       # resident pairs * P
    min_margin: float      # min distance of a resident score to the grid values that decide centre_bin


def thresholds_for_drop_rate(logits: np.ndarray, K: int, P: int, rate: float, offset_bins, lo: int = 0,
                             hi: Optional[int] = None, n_bins: int = 4096) -> DropRateThresholds:
    """The map from a target drop rate to thresholds (Sec. 5.3.3: the relation is not linear, so it
    is read off the batch's own score distribution; Sec. 4.2 c: the partitions' thresholds keep fixed
    offsets around a centre, e.g. -0.01 / +0.01).

    Thresholds live on the grid of multiples of 1/n_bins: tau_p = (b + offset_bins[p]) / n_bins.  b is
    the smallest integer for which at least rate * total_units units of the pairs routed to the
    resident experts [lo, hi) fall below their threshold (unit (pair, p) is dropped iff n < tau_p).
    Plain counting over the candidates, scores compared in single precision."""
    f32 = np.float32
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    T, E = logits.shape
    hi = E if hi is None else hi
    off = [int(v) for v in offset_bins]
    assert len(off) == P
    r = route(logits, K, P, np.zeros((E, P), np.float32))
    n = r.n.astype(np.float32)[(r.idx >= lo) & (r.idx < hi)]
    total = int(n.size) * P
    need = rate * total

    def dropped(b):
        return sum(int((n < f32(b + k) / f32(n_bins)).sum()) for k in off)

    b = -max(off)                        # every threshold <= 0: nothing can be dropped
    top = n_bins + 1 - min(off)          # every threshold > 1: everything is dropped
    while b < top and dropped(b) < need:
        b += 1
    tau = np.tile(np.array([f32(b + k) / f32(n_bins) for k in off], dtype=np.float32)[None, :], (E, 1))
    margin = np.inf
    if n.size:
        for k in off:
            for edge in (b + k, b - 1 + k):
                margin = min(margin, float(np.abs(n.astype(np.float64) - edge / n_bins).min()))
    return DropRateThresholds(tau, b, dropped(b), total, float(margin))
