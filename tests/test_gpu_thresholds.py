"""GPU parity of the on-device load-aware threshold selection (paper Sec. 4.3): the table
moe_select_thresholds writes must equal the oracle's bit for bit (fp32 arithmetic on both sides),
and feeding it to the layer must respect the row budget."""
import numpy as np
import pytest

from synth import LAYERS, make_logits
from gpu_util import to_dev, GUARD

pytestmark = pytest.mark.gpu


def make_layer_obj(E, K, P, T, lo=0, hi=None):
    from paper_2508_18376_amd import DualSparseLayer
    return DualSparseLayer(d_model=32, d_ff=32 * P, n_experts=E, top_k=K, n_part=P, max_tokens=max(T, 1), dtype="f32",
                           expert_lo=lo, expert_hi=E if hi is None else hi)


def skewed_logits(T, E, seed, skew):
    rng = np.random.default_rng(seed)
    lg = rng.standard_normal((T, E)).astype(np.float32)
    lg += (skew * np.log(1.0 / np.arange(1, E + 1) ** 1.2)).astype(np.float32)[None, :]
    return lg


def select_with_margin(oracle, logits, K, P, tau_max, G, cap):
    """Oracle selection; the row cap is nudged until no score sits within the guard band of the two
    grid values that decide the result (the GPU evaluates the scores in fp32)."""
    for c in range(cap, cap + 50):
        sel = oracle.select_thresholds(logits, K, P, tau_max, group_size=G, row_cap=c)
        if c == 0 or K == 1 or sel.min_margin > GUARD:  # K = 1: every score is exactly s/s = 1 on both sides
            return c, sel
    raise AssertionError("no row cap with a safe margin")


CASES = [
    # name, T, E, K, P, group, cap, skew
    ("ratio_only", 1000, 8, 2, 2, 1, 0, 1.0),
    ("ratio_groups", 1500, 16, 4, 2, 4, 0, 1.0),
    ("cap_small_E", 3000, 8, 2, 4, 1, 500, 1.0),
    ("cap_many_E", 4000, 64, 8, 2, 8, 300, 0.7),
    ("cap_balanced", 2000, 8, 2, 1, 2, 400, 0.0),
    ("cap_128_experts", 700, 128, 6, 2, 1, 20, 0.5),
    ("one_token", 1, 8, 2, 2, 1, 1, 0.0),
    ("top1_scores_are_one", 500, 4, 1, 2, 1, 60, 1.0),
]


@pytest.mark.parametrize("name,T,E,K,P,G,cap,skew", CASES, ids=[c[0] for c in CASES])
def test_selected_thresholds_equal_the_oracle(oracle, name, T, E, K, P, G, cap, skew):
    import torch
    logits = skewed_logits(T, E, 100 + T, skew)
    tau_max = np.linspace(0.10, 0.14, P).astype(np.float32) if P > 1 else np.float32([0.12])
    cap, sel = select_with_margin(oracle, logits, K, P, tau_max, G, cap)
    layer = make_layer_obj(E, K, P, T)
    tau, pairs = layer.select_thresholds(to_dev(logits), to_dev(tau_max), group_size=G, row_cap=cap)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(pairs.cpu().numpy(), sel.pair_count)
    np.testing.assert_array_equal(tau.cpu().numpy().view(np.uint32), sel.tau.view(np.uint32))
    # the table is what the layer consumes: routing with it keeps at most `cap` rows per expert
    if cap > 0:
        idx, w, keep, gc = layer.route_and_mask(to_dev(logits), tau)
        torch.cuda.synchronize()
        idx_h, keep_h = idx.cpu().numpy(), keep.cpu().numpy()
        for e in range(E):
            assert int((keep_h[idx_h == e] != 0).sum()) <= cap
    layer.close()


def test_empty_batch_and_bad_arguments(oracle):
    import torch
    from paper_2508_18376_amd import binding as ds
    layer = make_layer_obj(8, 2, 2, 16)
    tau_max = to_dev(np.float32([0.2, 0.3]))
    tau, pairs = layer.select_thresholds(torch.empty((0, 8), dtype=torch.float32, device="cuda"), tau_max, row_cap=3)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(tau.cpu().numpy(), np.tile(np.float32([0.2, 0.3]), (8, 1)))
    assert pairs.cpu().numpy().tolist() == [0] * 8
    lg = to_dev(np.zeros((4, 8), np.float32))
    with pytest.raises(RuntimeError):
        layer.select_thresholds(lg, tau_max, group_size=3)   # does not divide E
    with pytest.raises(RuntimeError):
        layer.select_thresholds(lg, tau_max, row_cap=-1)
    layer.close()


def test_full_size_olmoe_router(oracle):
    """C3's router (64 experts, top-8, full batch), eight experts per device, Zipf-skewed."""
    import torch
    spec = LAYERS["C3"]
    logits = make_logits(spec.with_(zipf_s=0.6))
    tau_max = np.float32([0.05, 0.07])
    cap, sel = select_with_margin(oracle, logits, spec.K, spec.P, tau_max, 8, int(1.1 * spec.T * spec.K / spec.E))
    layer = make_layer_obj(spec.E, spec.K, spec.P, spec.T)
    tau, pairs = layer.select_thresholds(to_dev(logits), to_dev(tau_max), group_size=8, row_cap=cap)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(pairs.cpu().numpy(), sel.pair_count)
    np.testing.assert_array_equal(tau.cpu().numpy().view(np.uint32), sel.tau.view(np.uint32))
    assert (sel.cap_bin > 0).any() and (sel.ratio < 1).any() and (sel.ratio > 1).any()
    layer.close()


DROP_CASES = [
    # name, T, E, K, P, window, rate, offsets
    ("one_threshold", 2000, 8, 2, 1, None, 0.25, [0]),
    ("two_thresholds", 3000, 8, 2, 2, None, 0.25, [-41, 41]),
    ("four_parts", 4096, 8, 2, 4, None, 0.5, [-41, -14, 14, 41]),
    ("fine_grained_window", 2500, 64, 8, 2, (8, 24), 0.3, [-41, 41]),
    ("many_experts", 600, 160, 6, 2, None, 0.1, [-20, 20]),
    ("drop_nothing", 500, 8, 2, 2, None, 0.0, [-41, 41]),
    ("drop_everything", 500, 8, 2, 2, None, 1.0, [-41, 41]),
]


@pytest.mark.parametrize("name,T,E,K,P,window,rate,offsets", DROP_CASES, ids=[c[0] for c in DROP_CASES])
def test_thresholds_for_a_target_drop_rate_equal_the_oracle(oracle, name, T, E, K, P, window, rate, offsets):
    import torch
    lo, hi = window if window else (0, E)
    for seed in range(200, 230):  # a batch whose scores keep clear of the deciding grid values
        logits = skewed_logits(T, E, seed, 0.5)
        ref = oracle.thresholds_for_drop_rate(logits, K, P, rate, offsets, lo=lo, hi=hi)
        if rate in (0.0, 1.0) or ref.min_margin > GUARD:
            break
    else:
        raise AssertionError("no batch with a safe margin")
    layer = make_layer_obj(E, K, P, T, lo=lo, hi=hi)
    tau, stats = layer.thresholds_for_drop_rate(to_dev(logits), rate, offsets)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(tau.cpu().numpy().view(np.uint32), ref.tau.view(np.uint32))
    assert stats.cpu().numpy().tolist() == [ref.dropped_units, ref.total_units]
    # the table does what it says when the layer's own mask uses it
    idx, w, keep, gc = layer.route_and_mask(to_dev(logits), tau)
    torch.cuda.synchronize()
    kept = int(gc.sum().item())
    assert ref.total_units - kept == ref.dropped_units
    if 0 < rate < 1:
        assert ref.dropped_units >= rate * ref.total_units > ref.dropped_units - P * max(1, T * K // 50)
    layer.close()


def test_default_offsets_spread_one_hundredth_each_way():
    import torch
    layer = make_layer_obj(8, 2, 4, 64)
    logits = to_dev(skewed_logits(64, 8, 1, 0.0))
    tau, _ = layer.thresholds_for_drop_rate(logits, 0.25)
    torch.cuda.synchronize()
    row = tau[0].cpu().numpy()
    np.testing.assert_allclose(np.diff(row), [27 / 4096, 28 / 4096, 27 / 4096], atol=1e-7)   # -41, -14, 14, 41 grid steps
    with pytest.raises(RuntimeError):
        layer.thresholds_for_drop_rate(logits, 1.5)
    layer.close()
