"""Pins for the fp64 oracle: closed forms, library special cases, invariants the paper states,
brute force on tiny inputs and the golden fixtures.  None of these needs a GPU.

Paper passages: Eq. 1-4 (Sec. 2.1.1), Sec. 3.1 (complete transformation), Sec. 3.2 (partial
transformation), Sec. 4.1 (1T-Drop), Sec. 4.2 (reconstruction, 2T-Drop), Sec. 5.4 (EES rule).
"""
import json
import math
import os

import numpy as np
import pytest
import scipy.special

from synth import LayerSpec, make_layer, f32_to_bf16_bits, bf16_bits_to_f32
from threshold_util import spread_thresholds

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def tiny(**kw):
    base = dict(name="tiny", T=5, D=8, F=8, E=4, K=2, P=2, dtype="f32", seed=11, x_std=1.0, w_std=0.5)
    base.update(kw)
    return LayerSpec(**base)


def tau_full(spec, v):
    v = np.asarray(v, dtype=np.float32)
    if v.ndim == 0:
        return np.full((spec.E, spec.P), float(v), dtype=np.float32)
    if v.ndim == 1:
        return np.tile(v[None, :], (spec.E, 1)).astype(np.float32)
    return v


def run(oracle, spec, t, tau, **kw):
    return oracle.forward(t["x"], t["logits"], t["w1"], t["w3"], t["w2"], tau_full(spec, tau), spec.K, spec.P,
                          perm=kw.pop("perm", t["perm"]), sh_w1=t.get("sh_w1"), sh_w3=t.get("sh_w3"),
                          sh_w2=t.get("sh_w2"), lo=spec.lo, hi=spec.hi, **kw)


def silu(a):
    return a / (1.0 + np.exp(-a))


def ffn64(x, w1, w3, w2):
    x, w1, w3, w2 = (np.asarray(v, dtype=np.float64) for v in (x, w1, w3, w2))
    return (silu(x @ w1) * (x @ w3)) @ w2


# ----------------------------------------------------------------------------- gating

def brute_topk(row, K):
    order = sorted(range(len(row)), key=lambda e: (-float(row[e]), e))
    return order[:K]


@pytest.mark.parametrize("E,K", [(8, 2), (64, 8), (5, 5), (1, 1), (3, 1)])
def test_topk_is_sort_by_value_then_index(oracle, E, K):
    rng = np.random.default_rng(E * 100 + K)
    logits = rng.standard_normal((200, E)).astype(np.float32)
    logits[::3] = np.round(logits[::3] * 2) / 2  # many exact ties
    logits[5] = 0.25                             # all equal
    r = oracle.route(logits, K, 1, np.zeros((E, 1), np.float32))
    for t in range(logits.shape[0]):
        assert list(r.idx[t]) == brute_topk(logits[t], K), t
    assert list(r.idx[5]) == list(range(K))


def test_topk_full_width_is_a_permutation_sorted_by_value(oracle):
    rng = np.random.default_rng(3)
    logits = rng.standard_normal((50, 7)).astype(np.float32)
    r = oracle.route(logits, 7, 1, np.zeros((7, 1), np.float32))
    for t in range(50):
        assert sorted(r.idx[t]) == list(range(7))
        v = logits[t][r.idx[t]]
        assert np.all(v[:-1] >= v[1:])
    # K = E: the selected scores are the whole softmax and sum to one
    np.testing.assert_allclose(r.s.sum(axis=1), 1.0, rtol=0, atol=1e-14)
    np.testing.assert_allclose(r.n, r.s, rtol=1e-14)


def test_scores_match_library_softmax_and_normalise_to_one(oracle):
    rng = np.random.default_rng(4)
    logits = (rng.standard_normal((300, 16)) * 3).astype(np.float32)
    K = 4
    r = oracle.route(logits, K, 1, np.zeros((16, 1), np.float32))
    sm = scipy.special.softmax(logits.astype(np.float64), axis=1)
    np.testing.assert_allclose(r.s, np.take_along_axis(sm, r.idx.astype(np.int64), axis=1), rtol=1e-13)
    np.testing.assert_allclose(r.n.sum(axis=1), 1.0, atol=1e-14)
    np.testing.assert_allclose(r.n, r.s / r.s.sum(axis=1, keepdims=True), rtol=1e-14)
    # combine weight: raw score by default, normalised score on request
    np.testing.assert_array_equal(r.g, r.s)
    r2 = oracle.route(logits, K, 1, np.zeros((16, 1), np.float32), renorm=True)
    np.testing.assert_array_equal(r2.g, r2.n)


def test_top2_closed_form_and_the_ln4_rule(oracle):
    """K = 2: n_2 = 1 / (1 + exp(l_(1) - l_(2))).  With tau = 0.2 the second slot is dropped iff
    the logit gap exceeds ln 4, and the first slot (n_1 >= 1/2) never is for tau <= 0.5."""
    rng = np.random.default_rng(0)
    logits = rng.standard_normal((2000, 8)).astype(np.float32)
    tau = np.full((8, 2), 0.2, np.float32)
    r = oracle.route(logits, 2, 2, tau)
    srt = np.sort(logits.astype(np.float64), axis=1)
    gap = srt[:, -1] - srt[:, -2]
    np.testing.assert_allclose(r.n[:, 1], 1.0 / (1.0 + np.exp(gap)), rtol=1e-13)
    assert np.all(r.keep[:, 0, :] == 1)
    far = np.abs(gap - math.log(4.0)) > 1e-4
    assert np.array_equal(r.keep[far, 1, 0] == 0, gap[far] > math.log(4.0))
    assert np.array_equal(r.keep[:, 1, 0], r.keep[:, 1, 1])


def test_threshold_equality_keeps_and_tau_above_one_drops_all(oracle):
    # K = 1: the normalised score is exactly 1; tau = 1 keeps (only scores strictly below drop)
    logits = np.random.default_rng(1).standard_normal((20, 4)).astype(np.float32)
    assert oracle.route(logits, 1, 2, np.full((4, 2), 1.0, np.float32)).keep.all()
    assert not oracle.route(logits, 1, 2, np.full((4, 2), 2.0, np.float32)).keep.any()
    # exact tie of two logits with E = K = 2: n = 0.5 exactly, tau = 0.5 keeps both
    tie = np.zeros((1, 2), np.float32)
    assert oracle.route(tie, 2, 1, np.full((2, 1), 0.5, np.float32)).keep.all()
    # tau = 0 keeps everything, even a score that underflows to zero
    wide = np.array([[0.0, -2000.0]], np.float32)
    r = oracle.route(wide, 2, 1, np.zeros((2, 1), np.float32))
    assert r.n[0, 1] == 0.0 and r.keep.all()


def test_golden_index_remap_and_group_counts(oracle):
    cases = json.load(open(os.path.join(GOLD, "index_remap.json")))["cases"]
    for c in cases:
        P, E, sel = c["P"], c["E"], c["selected"]
        K = len(sel)
        logits = np.full((1, E), -5.0, np.float32)
        for rank, e in enumerate(sel):
            logits[0, e] = 5.0 - rank  # selection order = listed order
        r = oracle.route(logits, K, P, np.zeros((E, P), np.float32))
        assert list(r.idx[0]) == sel
        # the kept units, listed partition-major as in the remap equation
        got = [int(r.idx[0, k]) * P + p for p in range(P) for k in range(K) if r.keep[0, k, p]]
        assert got == c["sub_experts"]
        want = np.zeros(E * P, np.int64)
        want[c["sub_experts"]] = 1
        np.testing.assert_array_equal(r.group_count, want)


def test_group_counts_recount(oracle):
    rng = np.random.default_rng(7)
    E, K, P = 16, 4, 3
    logits = rng.standard_normal((500, E)).astype(np.float32)
    tau = rng.uniform(0.1, 0.4, (E, P)).astype(np.float32)
    r = oracle.route(logits, K, P, tau, lo=2, hi=11)
    want = np.zeros(E * P, np.int64)
    for t in range(500):
        for k in range(K):
            for p in range(P):
                e = int(r.idx[t, k])
                kept = 2 <= e < 11 and np.float32(r.n[t, k]) >= tau[e, p]
                assert bool(r.keep[t, k, p]) == bool(kept)
                want[e * P + p] += int(kept)
    np.testing.assert_array_equal(r.group_count, want)
    assert r.group_count.sum() == r.keep.sum()
    bits = r.keep_bits
    assert bits.shape == (500, K) and int(bits.max()) < (1 << P)
    assert np.array_equal((bits >> 1) & 1, r.keep[:, :, 1])


def test_golden_two_threshold_cases(oracle):
    gold = json.load(open(os.path.join(GOLD, "two_threshold_cases.json")))
    from paper_2508_18376_amd.thresholds import dual_thresholds, offset_bins
    for pr in gold["printed_pairs"]:
        # the tests' own spread rule and the product's policy both reproduce the printed pairs
        for th in (spread_thresholds(pr["T1"], 2), dual_thresholds(pr["T1"], 2)):
            np.testing.assert_allclose(th, [pr["T_major"], pr["T_minor"]], atol=1e-7)
        # and so do the product's grid offsets (multiples of 2^-12) to within half a grid step
        np.testing.assert_allclose(pr["T1"] + np.array(offset_bins(2)) / 4096.0, [pr["T_major"], pr["T_minor"]], atol=0.5 / 4096)
    for c in gold["cases"]:
        n2 = c["n"]
        logits = np.array([[0.0, math.log(n2 / (1.0 - n2))]], np.float32)  # E = K = 2: scores (1-n2, n2)
        tau = np.tile(np.array([[c["T_major"], c["T_minor"]]], np.float32), (2, 1))
        r = oracle.route(logits, 2, 2, tau)
        assert list(r.idx[0]) == [0, 1]
        assert abs(r.n[0, 1] - n2) < 1e-7
        assert list(r.keep[0, 1]) == [c["keep_major"], c["keep_minor"]], c
        assert list(r.keep[0, 0]) == [1, 1]


def test_equal_thresholds_are_single_threshold_drop_and_monotone(oracle):
    rng = np.random.default_rng(9)
    E, K, P = 8, 3, 4
    logits = rng.standard_normal((400, E)).astype(np.float32)
    one = oracle.route(logits, K, 1, np.full((E, 1), 0.3, np.float32))
    eq = oracle.route(logits, K, P, np.full((E, P), 0.3, np.float32))
    for p in range(P):
        np.testing.assert_array_equal(eq.keep[:, :, p], one.keep[:, :, 0])
    lo_t = rng.uniform(0.1, 0.3, (E, P)).astype(np.float32)
    hi_t = lo_t + rng.uniform(0.0, 0.2, (E, P)).astype(np.float32)
    a = oracle.route(logits, K, P, lo_t).keep
    b = oracle.route(logits, K, P, hi_t).keep
    assert np.all(b <= a)


def test_ees_rule_is_a_threshold_on_the_normalised_score(oracle):
    """Top-2: 'skip the second expert if score_2 < beta * score_1' == n_2 < beta / (1 + beta)."""
    rng = np.random.default_rng(10)
    logits = rng.standard_normal((1000, 8)).astype(np.float32)
    beta = 0.37
    thr = beta / (1.0 + beta)
    r = oracle.route(logits, 2, 1, np.full((8, 1), thr, np.float32))
    safe = np.abs(r.n[:, 1] - thr) > 1e-6
    skip = r.s[:, 1] < beta * r.s[:, 0]
    assert np.array_equal(r.keep[safe, 1, 0] == 0, skip[safe])


def test_golden_complete_transformation_thresholds():
    rows = json.load(open(os.path.join(GOLD, "complete_transform_thresholds.json")))["rows"]
    base = rows[0]["T1"]
    for r in rows:
        assert abs(r["T1"] - base / r["P"]) <= 0.005 + 1e-12  # printed to two decimals


# ----------------------------------------------------------------------------- layer output

def test_single_expert_is_the_textbook_swiglu_ffn(oracle):
    spec = tiny(T=7, D=12, F=20, E=1, K=1, P=1)
    t = make_layer(spec)
    want = ffn64(t["x"], t["w1"][0][:, :], t["w3"][0], t["w2"][0])
    for renorm in (False, True):
        got = run(oracle, spec, t, 0.0, renorm=renorm)
        np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-14)


def dense_moe64(spec, t, g, idx):
    """Eq. 3 with library matmuls: y = sum_k g_k f_{e_k}(x)."""
    y = np.zeros((spec.T, spec.D))
    for e in range(spec.lo, spec.hi):
        fe = ffn64(t["x"], t["w1"][e - spec.lo], t["w3"][e - spec.lo], t["w2"][e - spec.lo])
        for k in range(spec.K):
            m = idx[:, k] == e
            y[m] += g[m, k][:, None] * fe[m]
    return y


@pytest.mark.parametrize("renorm", [False, True])
def test_no_drop_equals_dense_topk_moe(oracle, renorm):
    spec = tiny(T=40, D=16, F=24, E=6, K=3, P=1)
    t = make_layer(spec)
    r = oracle.route(t["logits"], spec.K, 1, np.zeros((spec.E, 1), np.float32), renorm=renorm)
    want = dense_moe64(spec, t, r.g, r.idx)
    got = run(oracle, spec, t, 0.0, renorm=renorm)
    np.testing.assert_allclose(got, want, rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("P", [2, 3, 4, 12])
def test_partition_without_drop_reproduces_the_layer(oracle, P):
    """sum_p f_{e,p}(x) = f_e(x); the partial transformation gives y^P = y (Sec. 3.2)."""
    spec1 = tiny(T=16, D=16, F=24, E=5, K=2, P=1)
    t = make_layer(spec1)
    y1 = run(oracle, spec1, t, 0.0)
    yp = run(oracle, spec1.with_(P=P), t, 0.0)
    np.testing.assert_allclose(yp, y1, rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("kind", ["identity", "reversed", "random"])
def test_neuron_order_is_irrelevant_without_drop(oracle, kind):
    spec = tiny(T=16, D=16, F=24, E=5, K=2, P=4, perm_kind=kind)
    t = make_layer(spec)
    y_perm = run(oracle, spec, t, 0.0)
    y_none = run(oracle, spec, t, 0.0, perm=None)
    np.testing.assert_allclose(y_perm, y_none, rtol=1e-12, atol=1e-14)


def test_drop_output_is_the_ffn_over_exactly_the_kept_neurons(oracle):
    """With drops, expert e contributes the SwiGLU sum over neurons {perm[e][j] : j in kept slices}."""
    spec = tiny(T=30, D=12, F=24, E=6, K=3, P=4, seed=21)
    t = make_layer(spec)
    rng = np.random.default_rng(5)
    tau = rng.uniform(0.15, 0.45, (spec.E, spec.P)).astype(np.float32)  # not monotone in p on purpose
    r = oracle.route(t["logits"], spec.K, spec.P, tau)
    assert 0 < r.keep.sum() < r.keep.size
    Fp = spec.F // spec.P
    want = np.zeros((spec.T, spec.D))
    x = t["x"].astype(np.float64)
    for tok in range(spec.T):
        for k in range(spec.K):
            e = int(r.idx[tok, k])
            kept = [int(t["perm"][e][j]) for p in range(spec.P) if r.keep[tok, k, p] for j in range(p * Fp, (p + 1) * Fp)]
            if not kept:
                continue
            w1 = t["w1"][e][:, kept]
            w3 = t["w3"][e][:, kept]
            w2 = t["w2"][e][kept, :]
            want[tok] += r.s[tok, k] * ffn64(x[tok:tok + 1], w1, w3, w2)[0]
    got = run(oracle, spec, t, tau)
    np.testing.assert_allclose(got, want, rtol=1e-11, atol=1e-13)


def test_full_drop_gives_zero_and_shared_experts_survive(oracle):
    spec = tiny(T=9, D=8, F=16, E=4, K=2, P=2)
    t = make_layer(spec)
    y = run(oracle, spec, t, 2.0)
    assert np.all(y == 0.0)
    spec_s = spec.with_(n_shared=2, F_sh=12)
    ts = make_layer(spec_s)
    ys = run(oracle, spec_s, ts, 2.0)
    want = sum(ffn64(ts["x"], ts["sh_w1"][s], ts["sh_w3"][s], ts["sh_w2"][s]) for s in range(2))
    np.testing.assert_allclose(ys, want, rtol=1e-12, atol=1e-14)
    # two shared experts are one expert of twice the width
    cat = dict(ts)
    cat["sh_w1"] = np.concatenate([ts["sh_w1"][0], ts["sh_w1"][1]], axis=1)[None]
    cat["sh_w3"] = np.concatenate([ts["sh_w3"][0], ts["sh_w3"][1]], axis=1)[None]
    cat["sh_w2"] = np.concatenate([ts["sh_w2"][0], ts["sh_w2"][1]], axis=0)[None]
    np.testing.assert_allclose(run(oracle, spec_s, cat, 0.2), run(oracle, spec_s, ts, 0.2), rtol=1e-12, atol=1e-14)


def test_layer_keeps_a_unit_whose_score_equals_the_threshold(oracle):
    # K = 1: n is exactly 1, so tau = 1 must behave like tau = 0 in the layer output too
    spec = tiny(T=6, D=8, F=8, E=3, K=1, P=2)
    t = make_layer(spec)
    y0 = run(oracle, spec, t, 0.0)
    assert np.abs(y0).max() > 0
    np.testing.assert_array_equal(run(oracle, spec, t, 1.0), y0)
    assert np.all(run(oracle, spec, t, np.nextafter(np.float32(1.0), np.float32(2.0))) == 0.0)


def test_dropping_removes_exactly_the_dropped_terms(oracle):
    """y(tau) = y(0) - sum over dropped units of g * (that sub-expert's output), each recomputed on its own."""
    spec = tiny(T=25, D=10, F=16, E=5, K=3, P=2, seed=31)
    t = make_layer(spec)
    tau = spread_thresholds(0.3, 2)
    r = oracle.route(t["logits"], spec.K, spec.P, tau_full(spec, tau))
    y0 = run(oracle, spec, t, 0.0)
    yt = run(oracle, spec, t, tau)
    Fp = spec.F // spec.P
    removed = np.zeros_like(y0)
    for tok in range(spec.T):
        for k in range(spec.K):
            e = int(r.idx[tok, k])
            for p in range(spec.P):
                if r.keep[tok, k, p]:
                    continue
                q = t["perm"][e][p * Fp:(p + 1) * Fp]
                removed[tok] += r.s[tok, k] * ffn64(t["x"][tok:tok + 1], t["w1"][e][:, q], t["w3"][e][:, q], t["w2"][e][q, :])[0]
    assert np.abs(removed).max() > 0
    np.testing.assert_allclose(yt, y0 - removed, rtol=1e-10, atol=1e-13)


def test_complete_transformation_gives_y_over_P(oracle):
    """Sec. 3.1: E*P experts with repeated router columns and Top-(K*P), W2 unscaled -> y / P;
    W2 scaled by P -> y.  Repeated logits are exact ties, so this also walks the tie rule."""
    spec = tiny(T=20, D=10, F=12, E=4, K=2, P=1, perm_kind="identity")
    t = make_layer(spec)
    y = run(oracle, spec, t, 0.0)
    for P in (2, 3):
        Fp = spec.F // P
        big = spec.with_(E=spec.E * P, K=spec.K * P, F=Fp)
        tb = {"x": t["x"], "logits": np.repeat(t["logits"], P, axis=1), "perm": None}
        tb["w1"] = np.stack([t["w1"][e][:, p * Fp:(p + 1) * Fp] for e in range(spec.E) for p in range(P)])
        tb["w3"] = np.stack([t["w3"][e][:, p * Fp:(p + 1) * Fp] for e in range(spec.E) for p in range(P)])
        tb["w2"] = np.stack([t["w2"][e][p * Fp:(p + 1) * Fp, :] for e in range(spec.E) for p in range(P)])
        rb = oracle.route(tb["logits"], big.K, 1, np.zeros((big.E, 1), np.float32))
        r1 = oracle.route(t["logits"], spec.K, 1, np.zeros((spec.E, 1), np.float32))
        want_idx = np.stack([r1.idx * P + p for p in range(P)], axis=2).reshape(spec.T, -1)  # e*P .. e*P+P-1 together
        np.testing.assert_array_equal(rb.idx, want_idx)
        np.testing.assert_allclose(rb.s, np.repeat(r1.s, P, axis=1) / P, rtol=1e-13)
        yb = run(oracle, big, tb, 0.0, perm=None)
        np.testing.assert_allclose(yb, y / P, rtol=1e-12, atol=1e-14)
        tb["w2"] = tb["w2"] * np.float32(P)
        if P == 2:  # scaling by a power of two is exact in float32
            np.testing.assert_allclose(run(oracle, big, tb, 0.0, perm=None), y, rtol=1e-12, atol=1e-14)


def test_resident_window_splits_the_sum_over_experts(oracle):
    spec = tiny(T=30, D=8, F=8, E=6, K=3, P=2, seed=41)
    t = make_layer(spec)
    tau = 0.25
    y_all = run(oracle, spec, t, tau)
    parts = []
    for lo, hi in ((0, 2), (2, 5), (5, 6)):
        sub = dict(t)
        for kname in ("w1", "w3", "w2", "perm"):
            sub[kname] = t[kname][lo:hi]
        parts.append(run(oracle, spec.with_(resident=(lo, hi)), sub, tau))
    np.testing.assert_allclose(sum(parts), y_all, rtol=1e-12, atol=1e-14)


def test_token_list_selects_rows(oracle):
    spec = tiny(T=20, D=8, F=8, E=4, K=2, P=2)
    t = make_layer(spec)
    y = run(oracle, spec, t, 0.3)
    pick = np.array([17, 0, 5, 5], np.int32)
    np.testing.assert_array_equal(run(oracle, spec, t, 0.3, tokens=pick), y[pick])
    with pytest.raises(ValueError):
        run(oracle, spec, t, 0.3, tokens=np.array([20], np.int32))


def test_bf16_inputs_are_widened_exactly(oracle):
    spec = tiny(T=10, D=16, F=16, E=4, K=2, P=2, dtype="bf16")
    t = make_layer(spec)
    wide = {k: (bf16_bits_to_f32(v) if v.dtype == np.uint16 else v) for k, v in t.items()}
    np.testing.assert_array_equal(run(oracle, spec, t, 0.3), run(oracle, spec, wide, 0.3))
    assert np.array_equal(f32_to_bf16_bits(wide["x"]), t["x"])


# ----------------------------------------------------------------------------- brute force

def brute_layer(spec, t, tau, renorm):
    """Independent pure-Python evaluation, one output element at a time (Eq. 1-4 + Sec. 4)."""
    T, D, F, E, K, P = spec.T, spec.D, spec.F, spec.E, spec.K, spec.P
    Fp = F // P
    y = [[0.0] * D for _ in range(T)]
    for tok in range(T):
        l = [float(v) for v in t["logits"][tok]]
        order = sorted(range(E), key=lambda e: (-l[e], e))[:K]
        mx = max(l)
        z = math.fsum(math.exp(v - mx) for v in l)
        s = [math.exp(l[e] - mx) / z for e in order]
        tot = math.fsum(s)
        n = [v / tot for v in s]
        x = [float(v) for v in t["x"][tok]]
        for d in range(D):
            terms = []
            for k, e in enumerate(order):
                if not (spec.lo <= e < spec.hi):
                    continue
                r = e - spec.lo
                g = n[k] if renorm else s[k]
                for p in range(P):
                    if np.float32(n[k]) < np.float32(tau[e][p]):
                        continue
                    for j in range(p * Fp, (p + 1) * Fp):
                        q = int(t["perm"][r][j])
                        a = math.fsum(x[i] * float(t["w1"][r][i][q]) for i in range(D))
                        b = math.fsum(x[i] * float(t["w3"][r][i][q]) for i in range(D))
                        terms.append(g * (a / (1.0 + math.exp(-a))) * b * float(t["w2"][r][q][d]))
            for sidx in range(spec.n_shared):
                for q in range(spec.F_sh):
                    a = math.fsum(x[i] * float(t["sh_w1"][sidx][i][q]) for i in range(D))
                    b = math.fsum(x[i] * float(t["sh_w3"][sidx][i][q]) for i in range(D))
                    terms.append((a / (1.0 + math.exp(-a))) * b * float(t["sh_w2"][sidx][q][d]))
            y[tok][d] = math.fsum(terms)
    return np.array(y)


GRID = [
    dict(T=1, D=8, F=8, E=1, K=1, P=1),
    dict(T=3, D=8, F=8, E=2, K=1, P=2),
    dict(T=3, D=8, F=8, E=2, K=2, P=4, perm_kind="reversed"),
    dict(T=4, D=8, F=8, E=8, K=2, P=2),
    dict(T=3, D=8, F=8, E=8, K=8, P=1, perm_kind="identity"),
    dict(T=3, D=6, F=12, E=5, K=3, P=3, n_shared=1, F_sh=5),
    dict(T=4, D=8, F=8, E=8, K=2, P=2, resident=(2, 6)),
]


@pytest.mark.parametrize("shape", GRID)
@pytest.mark.parametrize("tau_kind", ["zero", "0.2", "per_partition", "all"])
def test_brute_force_on_tiny_layers(oracle, shape, tau_kind):
    spec = tiny(seed=51, **shape)
    t = make_layer(spec)
    if tau_kind == "zero":
        tau = tau_full(spec, 0.0)
    elif tau_kind == "0.2":
        tau = tau_full(spec, 0.2)
    elif tau_kind == "all":
        tau = tau_full(spec, 2.0)
    else:
        tau = np.random.default_rng(1).uniform(0.05, 0.6, (spec.E, spec.P)).astype(np.float32)
    for renorm in (False, True):
        want = brute_layer(spec, t, tau, renorm)
        got = run(oracle, spec, t, tau, renorm=renorm)
        np.testing.assert_allclose(got, want, rtol=1e-11, atol=1e-13)


# ----------------------------------------------------------------------------- importance profiling

@pytest.mark.parametrize("metric", [0, 1, 2, 3])
def test_importance_single_expert_is_a_column_sum(oracle, metric):
    """E = K = 1: every token goes to the expert, so the metric is a plain column sum (Sec. 4.2 b)."""
    spec = tiny(T=23, D=12, F=20, E=1, K=1, P=1)
    t = make_layer(spec)
    x = t["x"].astype(np.float64)
    g = silu(x @ t["w1"][0].astype(np.float64))
    u = x @ t["w3"][0].astype(np.float64)
    want = {0: g, 1: np.abs(g), 2: g * u, 3: np.abs(g * u)}[metric].sum(axis=0)
    imp, ab = oracle.importance(t["x"], t["logits"], t["w1"], t["w3"], 1, metric)
    np.testing.assert_allclose(imp[0], want, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(ab[0], np.abs({0: g, 1: g, 2: g * u, 3: g * u}[metric]).sum(axis=0), rtol=1e-12)


def test_importance_counts_only_routed_tokens_and_orders_neurons(oracle):
    spec = tiny(T=60, D=10, F=16, E=5, K=2, P=1, seed=61)
    t = make_layer(spec)
    r = oracle.route(t["logits"], spec.K, 1, np.zeros((spec.E, 1), np.float32))
    x = t["x"].astype(np.float64)
    for metric in range(4):
        imp, ab = oracle.importance(t["x"], t["logits"], t["w1"], t["w3"], spec.K, metric)
        for e in range(spec.E):
            toks = np.nonzero((r.idx == e).any(axis=1))[0]
            g = silu(x[toks] @ t["w1"][e].astype(np.float64))
            u = x[toks] @ t["w3"][e].astype(np.float64)
            want = {0: g, 1: np.abs(g), 2: g * u, 3: np.abs(g * u)}[metric].sum(axis=0)
            np.testing.assert_allclose(imp[e], want, rtol=1e-11, atol=1e-13)
        if metric & 1:
            np.testing.assert_allclose(imp, ab, rtol=1e-14)
            assert np.all(imp >= 0)
        else:
            assert np.all(np.abs(imp) <= ab + 1e-15)
    # resident window = rows of the full result
    imp_all, _ = oracle.importance(t["x"], t["logits"], t["w1"], t["w3"], spec.K, 3)
    imp_win, _ = oracle.importance(t["x"], t["logits"], t["w1"][1:4], t["w3"][1:4], spec.K, 3, lo=1, hi=4)
    np.testing.assert_array_equal(imp_win, imp_all[1:4])
    # the permutation lists neurons by descending importance, equal values by ascending id
    tie = np.array([[0.5, 2.0, 0.5, 3.0, 2.0]])
    assert list(oracle.perm_from_importance(tie)[0]) == [3, 1, 4, 0, 2]
    perm = oracle.perm_from_importance(imp_all)
    for e in range(spec.E):
        assert sorted(perm[e]) == list(range(spec.F))
        assert np.all(np.diff(imp_all[e][perm[e]]) <= 0)


# ----------------------------------------------------------- load-aware thresholds (Sec. 4.3)
def _one_hot_logits(assign, E):
    """K = 1 routing by construction: token t goes to expert assign[t]."""
    lg = np.full((len(assign), E), -4.0, dtype=np.float32)
    lg[np.arange(len(assign)), assign] = 4.0
    return lg


def test_load_ratio_rule_on_a_hand_example(oracle):
    # pairs per expert 200, 100, 50, 50: ideal share 100 -> ratios 2, 1, 0.5, 0.5
    assign = np.repeat(np.arange(4), [200, 100, 50, 50])
    tau_max = np.array([0.25, 0.5], dtype=np.float32)
    sel = oracle.select_thresholds(_one_hot_logits(assign, 4), 1, 2, tau_max)
    np.testing.assert_array_equal(sel.pair_count, [200, 100, 50, 50])
    np.testing.assert_array_equal(sel.ratio, np.float32([2, 1, 0.5, 0.5]))
    np.testing.assert_array_equal(sel.tau, np.float32([[0.25, 0.5], [0.25, 0.5], [0.125, 0.25], [0.125, 0.25]]))
    # two experts per device: loads 300 and 100 against 200 -> ratios 1.5 and 0.5, shared by both experts of a device
    sel2 = oracle.select_thresholds(_one_hot_logits(assign, 4), 1, 2, tau_max, group_size=2)
    np.testing.assert_array_equal(sel2.ratio, np.float32([1.5, 0.5]))
    np.testing.assert_array_equal(sel2.tau, np.float32([[0.25, 0.5], [0.25, 0.5], [0.125, 0.25], [0.125, 0.25]]))
    # one device holding everything is balanced by definition
    sel3 = oracle.select_thresholds(_one_hot_logits(assign, 4), 1, 2, tau_max, group_size=4)
    np.testing.assert_array_equal(sel3.tau, np.tile(tau_max, (4, 1)))


def test_balanced_load_takes_the_maximum_threshold_everywhere(oracle):
    assign = np.tile(np.arange(8), 32)
    tau_max = np.array([0.11, 0.13, 0.17], dtype=np.float32)
    sel = oracle.select_thresholds(_one_hot_logits(assign, 8), 1, 3, tau_max)
    np.testing.assert_array_equal(sel.tau, np.tile(tau_max, (8, 1)))


def test_row_cap_threshold_is_the_grid_point_just_above_the_first_excluded_score(oracle):
    """Closed form of the cap: with v the (cap+1)-th largest score of the expert, at most cap scores
    are >= b/B exactly when b/B > v, so b = floor(v*B) + 1."""
    rng = np.random.default_rng(17)
    T, E, K, P, B = 600, 4, 2, 2, 4096
    logits = rng.standard_normal((T, E)).astype(np.float32)
    r = oracle.route(logits, K, P, np.zeros((E, P), np.float32))
    n32 = r.n.astype(np.float32)
    tau_max = np.array([0.02, 0.04], dtype=np.float32)
    for cap in (1, 37, 150):
        sel = oracle.select_thresholds(logits, K, P, tau_max, row_cap=cap, n_bins=B)
        base = oracle.select_thresholds(logits, K, P, tau_max, n_bins=B)
        for e in range(E):
            ne = np.sort(n32[r.idx == e])[::-1]
            assert ne.size > cap
            b = int(np.floor(float(ne[cap]) * B)) + 1
            assert sel.cap_bin[e] == b
            lifted = np.float32(b / B)
            assert lifted > base.tau[e, 0]
            np.testing.assert_array_equal(sel.tau[e], np.float32([lifted, lifted + (base.tau[e, 1] - base.tau[e, 0])]))
        # consequence, through the keep decision itself: the rows of every expert fit the cap, and the
        # next lower grid point would not
        rows = oracle.route(logits, K, P, sel.tau).keep.any(axis=2)
        lower = sel.tau - np.float32(1.0 / B)
        rows_lower = oracle.route(logits, K, P, lower).keep.any(axis=2)
        for e in range(E):
            assert rows[r.idx == e].sum() <= cap < rows_lower[r.idx == e].sum()


def test_row_cap_that_does_not_bind_changes_nothing_and_cap_edge_cases(oracle):
    rng = np.random.default_rng(18)
    logits = rng.standard_normal((300, 4)).astype(np.float32)
    tau_max = np.array([0.3, 0.32], dtype=np.float32)
    base = oracle.select_thresholds(logits, 2, 2, tau_max)
    loose = oracle.select_thresholds(logits, 2, 2, tau_max, row_cap=10_000)
    np.testing.assert_array_equal(loose.tau, base.tau)
    assert np.all(loose.cap_bin == 0)
    # K = 1: every score is exactly 1; a cap below the pair count can only be met above 1
    assign = np.repeat(np.arange(2), [30, 10])
    sel = oracle.select_thresholds(_one_hot_logits(assign, 2), 1, 1, np.float32([0.5]), row_cap=20, n_bins=1024)
    assert sel.cap_bin[0] == 1025 and sel.tau[0, 0] == np.float32(1025 / 1024)
    assert sel.cap_bin[1] == 0 and sel.tau[1, 0] == np.float32(0.5 * 0.5)
    assert oracle.route(_one_hot_logits(assign, 2), 1, 1, sel.tau).group_count.tolist() == [0, 10]


# ------------------------------------------- router GEMM and complete transformation (Sec. 3.1)
def test_router_logits_on_unit_vectors_and_bf16_widening(oracle):
    from synth import f32_to_bf16_bits
    wg = np.arange(12, dtype=np.float32).reshape(4, 3) - 5.0         # W_g [D=4][E=3]
    x = np.eye(4, dtype=np.float32)[[2, 0, 3]]                       # tokens e_2, e_0, e_3 pick rows of W_g
    np.testing.assert_array_equal(oracle.router_logits(x, wg), wg[[2, 0, 3]].astype(np.float64))
    x2 = np.float32([[1, 2, 3, 4], [0.5, -1, 0, 2]])
    want = [[sum(float(x2[t, d]) * float(wg[d, e]) for d in range(4)) for e in range(3)] for t in range(2)]
    np.testing.assert_array_equal(oracle.router_logits(x2, wg), np.float64(want))
    # bf16 storage: values are the bit patterns widened exactly
    np.testing.assert_array_equal(oracle.router_logits(f32_to_bf16_bits(x2), f32_to_bf16_bits(wg)), np.float64(want))


@pytest.mark.parametrize("P,dtype", [(2, "f32"), (4, "f32"), (2, "bf16"), (3, "f32")])
def test_complete_transform_function_preserves_the_layer(oracle, P, dtype):
    """The transformed layer (E*P experts, Top-(K*P), router columns repeated, W2 * P) computes the
    original layer's output (Sec. 3.1, last equation); without the W2 scaling it computes y / P."""
    from synth import make_router
    spec = tiny(T=24, D=16, F=24, E=4, K=2, P=1, dtype=dtype, seed=77, perm_kind="random", x_std=1.0, w_std=0.2)
    t = make_layer(spec)
    wg = make_router(spec)
    logits = oracle.router_logits(t["x"], wg).astype(np.float32)
    tau0 = np.zeros((spec.E, 1), np.float32)
    y = oracle.forward(t["x"], logits, t["w1"], t["w3"], t["w2"], tau0, spec.K, 1)
    wg_t, w1_t, w3_t, w2_t = oracle.complete_transform(wg, t["w1"], t["w3"], t["w2"], P, perm=t["perm"])
    assert wg_t.shape == (spec.D, spec.E * P) and w1_t.shape == (spec.E * P, spec.D, spec.F // P)
    logits_t = oracle.router_logits(t["x"], wg_t).astype(np.float32)
    np.testing.assert_array_equal(logits_t, np.repeat(logits, P, axis=1))
    tau0_t = np.zeros((spec.E * P, 1), np.float32)
    y_t = oracle.forward(t["x"], logits_t, w1_t, w3_t, w2_t, tau0_t, spec.K * P, 1)
    if P in (2, 4):  # exact scaling
        np.testing.assert_allclose(y_t, y, rtol=1e-11, atol=1e-13)
    else:            # W2 * 3 is rounded to the storage type: 2^-24 relative per weight
        np.testing.assert_allclose(y_t, y, rtol=0, atol=2e-7 * np.abs(y).max())
    _, _, _, w2_plain = oracle.complete_transform(wg, t["w1"], t["w3"], t["w2"], P, perm=t["perm"], scale_w2=False)
    y_p = oracle.forward(t["x"], logits_t, w1_t, w3_t, w2_plain, tau0_t, spec.K * P, 1)
    np.testing.assert_allclose(y_p, y / P, rtol=1e-11, atol=1e-13)


def test_complete_transform_places_the_permuted_neurons(oracle):
    """New expert e*P+p holds original neurons perm[e][p*F/P ..], in that order, in all three matrices."""
    rng = np.random.default_rng(5)
    E, D, F, P = 2, 3, 6, 3
    w1 = rng.standard_normal((E, D, F)).astype(np.float32)
    w3 = rng.standard_normal((E, D, F)).astype(np.float32)
    w2 = rng.standard_normal((E, F, D)).astype(np.float32)
    wg = rng.standard_normal((D, E)).astype(np.float32)
    perm = np.int32([[5, 0, 3, 1, 4, 2], [2, 3, 4, 5, 0, 1]])
    wg_t, w1_t, w3_t, w2_t = oracle.complete_transform(wg, w1, w3, w2, P, perm=perm)
    np.testing.assert_array_equal(wg_t[:, [0, 1, 2]], np.repeat(wg[:, :1], 3, axis=1))
    assert w1_t[1, 2, 0] == w1[0, 2, 3] and w1_t[1, 2, 1] == w1[0, 2, 1]      # expert 0, part 1: neurons 3, 1
    assert w3_t[5, 0, 1] == w3[1, 0, 1]                                        # expert 1, part 2: neurons 0, 1
    assert w2_t[2, 0, 1] == np.float32(3) * w2[0, 4, 1]                        # expert 0, part 2: neurons 4, 2; times P
    assert w2_t[3, 1, 2] == np.float32(3) * w2[1, 3, 2]


def test_thresholds_of_the_transformed_layer_are_the_originals_over_P(oracle):
    """In the transformed layer every normalised score is n / P (Sec. 3.1: s_{e,p} = s_e / P), so a
    single threshold tau on the original layer is tau / P there (Table 1 uses such values)."""
    from synth import make_router
    spec = tiny(T=200, D=16, F=8, E=8, K=2, P=1, seed=78, x_std=1.0)
    t = make_layer(spec, weights=False)
    logits = oracle.router_logits(t["x"], make_router(spec)).astype(np.float32)
    P = 2
    r = oracle.route(logits, spec.K, 1, np.full((spec.E, 1), 0.3, np.float32))
    rt = oracle.route(np.repeat(logits, P, axis=1), spec.K * P, 1, np.full((spec.E * P, 1), 0.3 / P, np.float32))
    assert min(r.min_margin, rt.min_margin) > 1e-9
    np.testing.assert_array_equal(rt.keep[:, :, 0], np.repeat(r.keep[:, :, 0], P, axis=1))
    np.testing.assert_allclose(rt.n, np.repeat(r.n, P, axis=1) / P, rtol=1e-12)


# ------------------------------------------------ drop rate -> thresholds (Sec. 5.3.3, Sec. 4.2 c)
def test_drop_rate_thresholds_follow_the_order_statistics(oracle):
    """One partition: dropping at least a fraction `rate` of m scores needs the threshold just above
    the ceil(rate*m)-th smallest score v: b = floor(v*B) + 1 (closed form, not the counting loop)."""
    rng = np.random.default_rng(23)
    T, E, K, B = 500, 8, 2, 4096
    logits = rng.standard_normal((T, E)).astype(np.float32)
    r = oracle.route(logits, K, 1, np.zeros((E, 1), np.float32))
    n32 = np.sort(r.n.astype(np.float32).ravel())
    for rate in (0.1, 0.25, 0.5, 0.9):
        res = oracle.thresholds_for_drop_rate(logits, K, 1, rate, [0], n_bins=B)
        need = int(np.ceil(rate * n32.size))
        v = float(n32[need - 1])
        assert res.centre_bin == int(np.floor(v * B)) + 1
        assert res.total_units == n32.size and res.dropped_units >= need
        # one grid step lower drops too little; the keep decision itself agrees with the count
        keep = oracle.route(logits, K, 1, res.tau).keep
        assert int((keep == 0).sum()) == res.dropped_units
        lower = oracle.route(logits, K, 1, res.tau - np.float32(1.0 / B)).keep
        assert int((lower == 0).sum()) < need


def test_drop_rate_thresholds_with_partition_offsets_and_window(oracle):
    rng = np.random.default_rng(24)
    T, E, K, P, B = 400, 8, 2, 2, 4096
    logits = rng.standard_normal((T, E)).astype(np.float32)
    res = oracle.thresholds_for_drop_rate(logits, K, P, 0.3, [-41, 41], lo=2, hi=6, n_bins=B)
    # the two thresholds are 82 grid steps (~0.02) apart, the same for every expert
    assert np.all(res.tau == res.tau[0]) and res.tau[0, 1] - res.tau[0, 0] == np.float32(82 / B)
    rr = oracle.route(logits, K, P, res.tau, lo=2, hi=6)
    resident = (rr.idx >= 2) & (rr.idx < 6)
    assert res.total_units == int(resident.sum()) * P
    dropped = int((rr.keep[resident] == 0).sum())
    assert dropped == res.dropped_units and dropped >= 0.3 * res.total_units
    one_less = oracle.route(logits, K, P, res.tau - np.float32(1.0 / B), lo=2, hi=6)
    assert int((one_less.keep[resident] == 0).sum()) < 0.3 * res.total_units
    # extremes: rate 0 drops nothing (thresholds <= 0), rate 1 drops everything (thresholds > 1)
    r0 = oracle.thresholds_for_drop_rate(logits, K, P, 0.0, [-41, 41], n_bins=B)
    assert r0.dropped_units == 0 and np.all(r0.tau <= 0)
    r1 = oracle.thresholds_for_drop_rate(logits, K, P, 1.0, [-41, 41], n_bins=B)
    assert r1.dropped_units == r1.total_units and np.all(r1.tau[:, 0] > 0.9)
