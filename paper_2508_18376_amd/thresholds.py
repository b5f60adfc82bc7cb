"""Host-side threshold policies that feed the `tau` table of the library (numpy only).

The library takes an explicit table tau[E][P]; how it is chosen is policy:
  - dual_thresholds: T_major = T - 0.01, T_minor = T + 0.01 around a single-threshold value
    (DualSparse-MoE Sec. 4.2 c), spread evenly when there are more than two partitions;
  - tau_for_drop_rate: the threshold <-> drop-rate map is not linear (Sec. 5.3.3), so a target
    rate is turned into a threshold through the empirical quantile of the normalised scores;
  - load_aware: per-expert (per-device) thresholds from the ratio of actual to ideal load
    (Sec. 4.3): ratio >= 1 -> the maximum threshold, ratio < 1 -> reduced in proportion.
"""
from __future__ import annotations

import numpy as np


def dual_thresholds(tau: float, P: int, delta: float = 0.01) -> np.ndarray:
    if P == 1:
        return np.array([tau], dtype=np.float32)
    p = np.arange(P, dtype=np.float64)
    return (tau + delta * (2 * p - (P - 1)) / (P - 1)).astype(np.float32)


GRID = 4096  # the library's on-device threshold selection works on multiples of 2^-12


def offset_bins(P: int, delta: float = 0.01) -> list:
    """dual_thresholds' offsets around the centre in steps of the library's threshold grid (0.01 = 41
    steps): the `offset_bins` argument of moe_thresholds_for_drop_rate."""
    return [int(round(float(v) * GRID)) for v in dual_thresholds(0.0, P, delta).astype(np.float64)]


def tau_for_drop_rate(n: np.ndarray, P: int, rate: float, window: float = 0.005, delta: float = 0.01) -> np.ndarray:
    """Per-partition thresholds dropping about `rate` of the (pair, partition) units.

    n: normalised scores of the candidate pairs (any shape).  Among the gaps between adjacent
    order statistics within +-window of the target quantile, the centre is put where all P
    thresholds are farthest from any score, so that fp32 rounding of n cannot flip a decision."""
    if rate <= 0:
        return np.zeros(P, dtype=np.float32)
    flat = np.sort(np.asarray(n, dtype=np.float64).ravel())
    m = flat.size
    lo = max(int((rate - window) * m), 1)
    hi = max(min(int((rate + window) * m), m - 1), lo)
    cand = 0.5 * (flat[lo - 1:hi] + flat[lo:hi + 1])
    off = dual_thresholds(0.0, P, delta).astype(np.float64)[None, :]
    th = (cand[:, None] + off).astype(np.float32).astype(np.float64)
    pos = np.searchsorted(flat, th.ravel()).reshape(th.shape)
    up = np.abs(flat[np.clip(pos, 0, m - 1)] - th)
    dn = np.abs(flat[np.clip(pos - 1, 0, m - 1)] - th)
    best = int(np.argmax(np.minimum(up, dn).min(axis=1)))
    return th[best].astype(np.float32)


def load_aware(pairs_per_expert: np.ndarray, tau_max: np.ndarray) -> np.ndarray:
    """tau[e][p] = tau_max[p] if load ratio r_e >= 1 else tau_max[p] * r_e, r_e = pairs_e / mean pairs."""
    pairs = np.asarray(pairs_per_expert, dtype=np.float64)
    r = pairs / max(pairs.mean(), 1e-30)
    scale = np.minimum(r, 1.0)
    return (scale[:, None] * np.asarray(tau_max, dtype=np.float64)[None, :]).astype(np.float32)


def tau_capping_rows(n_expert: np.ndarray, P: int, cap_rows: int, delta: float = 0.01) -> np.ndarray:
    """Smallest thresholds for one expert that keep at most cap_rows * P units of it.

    n_expert: normalised scores of the pairs routed to that expert."""
    m = int(np.asarray(n_expert).size)
    if m <= cap_rows:
        return np.zeros(P, dtype=np.float32)
    return tau_for_drop_rate(n_expert, P, 1.0 - cap_rows / m, window=min(0.005, 0.25 * cap_rows / m), delta=delta)
