"""GPU parity, layer output: moe_dualsparse_forward (through the C ABI) against the fp64 oracle,
element by element, on seeded layers small enough for the oracle but spanning several row tiles,
ragged tails, empty experts, fully dropped tokens, shared experts and a resident window.

Tolerances (relative to the RMS of the oracle output): fp32 layers 1e-5, bf16 layers 2e-2.
"""
import numpy as np
import pytest

from synth import LayerSpec, LAYERS, make_layer
from threshold_util import spread_thresholds
from gpu_util import GUARD, make_gpu_layer, to_dev, to_host64, pick_tau, tau_table, rel_err, assert_output_close, TOL

pytestmark = pytest.mark.gpu



def spec_of(**kw):
    base = dict(name="f", T=300, D=128, F=256, E=4, K=2, P=2, dtype="bf16", seed=7, x_std=1.0, w_std=0.02)
    base.update(kw)
    return LayerSpec(**base)


def oracle_forward(oracle, spec, t, tau, renorm=False, tokens=None):
    return oracle.forward(t["x"], t["logits"], t["w1"], t["w3"], t["w2"], tau, spec.K, spec.P, perm=t["perm"],
                          sh_w1=t.get("sh_w1"), sh_w3=t.get("sh_w3"), sh_w2=t.get("sh_w2"), lo=spec.lo, hi=spec.hi,
                          renorm=renorm, tokens=tokens)


def resolve_tau(oracle, spec, t, tau_kind):
    if isinstance(tau_kind, str) and tau_kind.startswith("rate"):
        r0 = oracle.route(t["logits"], spec.K, spec.P, np.zeros((spec.E, spec.P), np.float32), spec.lo, spec.hi)
        return tau_table(spec, pick_tau(r0.n, spec.P, float(tau_kind[4:])))
    if isinstance(tau_kind, str) and tau_kind == "ragged":
        # thresholds that are NOT monotone in p and differ per expert: general keep patterns
        # (re-drawn until no score sits inside the guard band)
        for attempt in range(50):
            rng = np.random.default_rng(spec.seed + 100 + attempt)
            tau = rng.uniform(0.05, 0.6, (spec.E, spec.P)).astype(np.float32)
            if oracle.route(t["logits"], spec.K, spec.P, tau, spec.lo, spec.hi).min_margin > 2 * GUARD:
                return tau
        raise AssertionError("no guard-band-free thresholds found")
    return tau_table(spec, tau_kind)


def run_case(oracle, spec, tau_kind, renorm=False, expect_mfma=None, tall_items=0):
    import torch
    t = make_layer(spec)
    tau = resolve_tau(oracle, spec, t, tau_kind)
    ref_r = oracle.route(t["logits"], spec.K, spec.P, tau, spec.lo, spec.hi, renorm=renorm)
    if ref_r.keep.size and 0 < ref_r.keep.sum() < ref_r.keep.size and spec.K > 1:
        assert ref_r.min_margin > GUARD, ref_r.min_margin
    y_ref = oracle_forward(oracle, spec, t, tau, renorm=renorm)
    layer, dev = make_gpu_layer(spec, t, renorm=renorm, tall_items=tall_items)
    if expect_mfma is not None:
        assert layer.uses_mfma == expect_mfma
    y = layer.forward(dev["x"], dev["logits"], to_dev(tau))
    torch.cuda.synchronize()
    y = to_host64(y, spec.dtype)
    assert_output_close(y, y_ref, spec.dtype)
    # tokens whose every unit is dropped (and no shared expert) are exact zeros
    if spec.n_shared == 0:
        dead = ref_r.keep.reshape(spec.T, -1).sum(axis=1) == 0
        assert np.all(y[dead] == 0.0)
    plan = layer.plan(spec.T)
    layer.close()
    return y, y_ref, ref_r, plan


# ---------------------------------------------------------------------------------- fp32 layers
@pytest.mark.parametrize("perm_kind", ["identity", "random"])
@pytest.mark.parametrize("tau_kind", ["one", "two"])
@pytest.mark.parametrize("renorm", [False, True])
def test_config1_fp32(oracle, perm_kind, tau_kind, renorm):
    spec = LAYERS["C1"].with_(perm_kind=perm_kind)
    tau = 0.2 if tau_kind == "one" else spread_thresholds(0.2, 2)
    run_case(oracle, spec, tau, renorm=renorm, expect_mfma=False)


F32_CASES = [
    ("ragged_shapes", spec_of(dtype="f32", T=131, D=72, F=120, E=5, K=3, P=3, x_std=0.5, w_std=0.1), "rate0.3"),
    ("tiny", spec_of(dtype="f32", T=1, D=8, F=8, E=1, K=1, P=1, x_std=1.0, w_std=0.5), 0.0),
    ("odd_D", spec_of(dtype="f32", T=33, D=7, F=10, E=3, K=2, P=2, x_std=1.0, w_std=0.5), "rate0.25"),
    ("shared", spec_of(dtype="f32", T=70, D=40, F=48, E=6, K=2, P=2, n_shared=2, F_sh=20, x_std=0.5, w_std=0.1), "rate0.25"),
    ("window", spec_of(dtype="f32", T=90, D=32, F=32, E=8, K=2, P=4, resident=(2, 5), x_std=0.5, w_std=0.1), "rate0.25"),
    ("general_masks", spec_of(dtype="f32", T=200, D=32, F=64, E=4, K=3, P=4, x_std=0.5, w_std=0.1), "ragged"),
    ("P8", spec_of(dtype="f32", T=150, D=32, F=64, E=4, K=2, P=8, x_std=0.5, w_std=0.1), "ragged"),
    ("all_dropped", spec_of(dtype="f32", T=40, D=32, F=32, E=4, K=2, P=2, x_std=0.5, w_std=0.1), 2.0),
    ("empty_experts", spec_of(dtype="f32", T=3, D=32, F=32, E=16, K=2, P=2, x_std=0.5, w_std=0.1), 0.0),
]


@pytest.mark.parametrize("name,spec,tau_kind", F32_CASES, ids=[c[0] for c in F32_CASES])
def test_fp32_generic_path(oracle, name, spec, tau_kind):
    y, y_ref, r, plan = run_case(oracle, spec, tau_kind, expect_mfma=False)
    if name == "all_dropped":
        assert np.all(y == 0.0)


# ---------------------------------------------------------------------------------- bf16 layers
BF16_CASES = [
    # several 256-row tiles per expert with ragged tails; 2 neuron tiles per partition; 2 K steps
    ("multi_tile", spec_of(T=1500, D=128, F=512, E=4, K=2, P=2), "rate0.25", True),
    ("no_drop", spec_of(T=700, D=256, F=256, E=4, K=2, P=2, seed=8), 0.0, True),
    ("half_drop_P4", spec_of(T=900, D=128, F=512, E=4, K=2, P=4, seed=9), "rate0.5", True),
    ("fine_grained", spec_of(T=600, D=128, F=128, E=16, K=4, P=2, seed=10), "rate0.25", True),
    ("Fp_704_like", spec_of(T=400, D=128, F=384, E=4, K=2, P=2, seed=11), "rate0.33", True),  # Fp=192: half-empty neuron tile
    # full row tiles under a last neuron tile that is half full (Fp = 192) or a quarter full (Fp = 160)
    ("half_neuron_tile", spec_of(T=1400, D=128, F=384, E=4, K=2, P=2, seed=24), "rate0.25", True),
    ("quarter_neuron_tile", spec_of(T=1200, D=192, F=320, E=4, K=2, P=2, seed=25), 0.0, True),
    ("shared", spec_of(T=500, D=128, F=256, E=8, K=2, P=2, n_shared=2, F_sh=192, seed=12), "rate0.33", True),
    ("window", spec_of(T=800, D=128, F=256, E=8, K=2, P=4, resident=(1, 3), seed=13), "rate0.25", True),
    ("general_masks", spec_of(T=700, D=128, F=512, E=4, K=3, P=4, seed=14), "ragged", True),
    ("P8", spec_of(T=500, D=64, F=512, E=4, K=2, P=8, seed=15), "ragged", True),
    ("all_dropped", spec_of(T=300, D=64, F=128, E=4, K=2, P=2, seed=16), 2.0, True),
    ("empty_experts", spec_of(T=3, D=64, F=128, E=16, K=2, P=2, seed=17), 0.0, True),
    ("one_token", spec_of(T=1, D=64, F=64, E=2, K=1, P=1, seed=18), 0.0, True),
    ("D_wider_than_tile", spec_of(T=300, D=320, F=128, E=4, K=2, P=2, seed=19), "rate0.25", True),
    ("generic_fallback", spec_of(T=200, D=72, F=80, E=4, K=2, P=2, seed=20), "rate0.25", False),
    # the limits of the configuration at once: 512 experts, top-16, 8 parts
    ("many_tokens", spec_of(T=70001, D=64, F=128, E=8, K=2, P=2, seed=23), "rate0.25", True),  # > 1024 row tiles, > 1000 route blocks
    # 64-row tiles on the generic path: > 2048 row tiles, whose keep patterns no longer fit the plan kernel's LDS
    ("many_tiles_generic", spec_of(T=70001, D=40, F=48, E=8, K=2, P=2, seed=26), "rate0.25", False),
    ("max_experts_topk_parts", spec_of(T=300, D=32, F=256, E=512, K=16, P=8, seed=22), "rate0.25", True),
]


@pytest.mark.parametrize("name,spec,tau_kind,mfma", BF16_CASES, ids=[c[0] for c in BF16_CASES])
def test_bf16_layers(oracle, name, spec, tau_kind, mfma):
    y, y_ref, r, plan = run_case(oracle, spec, tau_kind, expect_mfma=mfma)
    if name == "all_dropped":
        assert np.all(y == 0.0)


# The matrix-core path keeps the intermediate activation in half precision and W2 as half precision
# times a power of two chosen from the largest |W2|: layers whose weights or activations are far from
# the synthetic layers' scale must come out as exactly as those.
SCALE_CASES = [
    # (name, weight std, activation std, cfg.h_scale_log2)
    ("large_weights", 0.6, 1.0, 0),        # |W2| up to ~3; activations of a few hundred
    ("tiny_weights", 2e-3, 1.0, 0),        # |W2| ~ 1e-2 at most, far below half precision's normal range unscaled
    ("tiny_activations", 0.02, 0.02, 14),  # h ~ 1e-5: below half precision's normal range unless centred by 2^14
    ("huge_activations", 0.5, 40.0, -12),  # h up to ~1e6: beyond 65504 unless scaled down
]


@pytest.mark.parametrize("name,w_std,x_std,k", SCALE_CASES, ids=[c[0] for c in SCALE_CASES])
def test_weight_and_activation_scales_far_from_one(oracle, name, w_std, x_std, k):
    import torch
    spec = spec_of(T=600, D=256, F=512, E=4, K=2, P=2, seed=31, w_std=w_std, x_std=x_std)
    t = make_layer(spec)
    tau = resolve_tau(oracle, spec, t, "rate0.25")
    y_ref = oracle_forward(oracle, spec, t, tau)
    for y_fp32 in (True, False):
        layer, dev = make_gpu_layer(spec, t, y_fp32=y_fp32, h_scale_log2=k)
        assert layer.uses_mfma
        y = layer.forward(dev["x"], dev["logits"], to_dev(tau))
        torch.cuda.synchronize()
        err = assert_output_close(to_host64(y, "f32" if y_fp32 else "bf16"), y_ref, "bf16", y_fp32=y_fp32)
        if y_fp32:
            assert err < 5e-3, err  # the computation itself is an order of magnitude inside the bar
        layer.close()


@pytest.mark.parametrize("name", ["fine_grained_K8", "shared_split_k"])
def test_partial_outputs_in_fp32_and_in_half_precision(oracle, name):
    """cfg.partial_fp32: both settings meet the bar (the fp32 output shows the computation's own error),
    and fp32 partials are at least as close to the oracle as half-precision ones."""
    import torch
    spec = (spec_of(T=900, D=256, F=256, E=16, K=8, P=2, seed=41) if name == "fine_grained_K8"
            else spec_of(T=40, D=512, F=2048, E=4, K=2, P=2, n_shared=1, F_sh=512, seed=42))  # few row tiles: K split in GEMM-2
    t = make_layer(spec)
    tau = resolve_tau(oracle, spec, t, "rate0.25")
    y_ref = oracle_forward(oracle, spec, t, tau)
    err = {}
    for partial_fp32 in (False, True):
        layer, dev = make_gpu_layer(spec, t, y_fp32=True, partial_fp32=partial_fp32)
        assert layer.uses_mfma
        y = layer.forward(dev["x"], dev["logits"], to_dev(tau))
        torch.cuda.synchronize()
        err[partial_fp32] = assert_output_close(to_host64(y, "f32"), y_ref, "bf16", y_fp32=True)
        if name == "shared_split_k":
            assert int(layer.plan(spec.T)["counters"][3]) > 1
        layer.close()
    assert err[False] < 5e-3 and err[True] <= err[False] * 1.05, err


def test_partition_and_reorder_invariance_on_gpu(oracle):
    """No drop: the output must not depend on P or on the neuron order (paper Sec. 3.2 identity);
    checked GPU-against-oracle for each variant, and the oracle outputs agree among themselves."""
    base = spec_of(dtype="f32", T=50, D=32, F=48, E=4, K=2, P=1, x_std=0.5, w_std=0.1, perm_kind="identity")
    t = make_layer(base)
    y1 = oracle_forward(oracle, base, t, tau_table(base, 0.0))
    for P, kind in ((2, "random"), (4, "reversed"), (8, "random")):
        spec = base.with_(P=P, perm_kind=kind)
        y, y_ref, _, _ = run_case(oracle, spec, 0.0)
        assert rel_err(y_ref, y1) < 1e-12
        assert rel_err(y, y1) <= TOL["f32"]


# ---------------------------------------------------------------------------------- row lists
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_row_lists_match_oracle_as_sets(oracle, dtype):
    spec = spec_of(dtype=dtype, T=1100, D=64, F=256, E=6, K=3, P=4, seed=21, resident=(1, 5))
    y, y_ref, r, plan = run_case(oracle, spec, "ragged")
    bits_ref = r.keep_bits
    np.testing.assert_array_equal(plan["topk_idx"].cpu().numpy(), r.idx)
    np.testing.assert_array_equal(plan["keep_bits"].cpu().numpy(), bits_ref)
    row_token = plan["row_token"].cpu().numpy()
    row_bits = plan["row_bits"].cpu().numpy()
    pair_row = plan["pair_row"].cpu().numpy()
    nrows = plan["expert_nrows"].cpu().numpy()
    row0 = plan["expert_row0"].cpu().numpy()
    BM = plan["tile_rows"]
    seen_rows = set()
    for i, e in enumerate(range(spec.lo, spec.hi)):
        want = sorted((int(tok), int(bits_ref[tok, k])) for tok in range(spec.T) for k in range(spec.K)
                      if r.idx[tok, k] == e and bits_ref[tok, k])
        assert nrows[i] == len(want)
        assert row0[i] % BM == 0
        rows = range(row0[i], row0[i] + nrows[i])
        got = sorted((int(row_token[q]), int(row_bits[q])) for q in rows)
        assert got == want
        # rows are grouped by keep pattern, patterns that keep partition 0 first
        key = [int("".join(str((int(row_bits[q]) >> p) & 1) for p in range(min(spec.P, 4))), 2) for q in rows]
        assert key == sorted(key, reverse=True)
        seen_rows.update(rows)
    # pair -> row is the inverse map; dropped or non-resident pairs have no row
    for tok in range(spec.T):
        for k in range(spec.K):
            q = int(pair_row[tok, k])
            if bits_ref[tok, k]:
                assert q in seen_rows and row_token[q] == tok and row_bits[q] == bits_ref[tok, k]
            else:
                assert q == -1
    assert len(set(pair_row[pair_row >= 0].tolist())) == int((pair_row >= 0).sum())


# ---------------------------------------------------------------------------------- error paths
def test_bad_permutation_is_rejected():
    import torch
    from paper_2508_18376_amd import DualSparseLayer, DsmoeError
    spec = spec_of(dtype="f32", T=8, D=16, F=16, E=2, K=1, P=2)
    t = make_layer(spec)
    layer = DualSparseLayer(d_model=16, d_ff=16, n_experts=2, top_k=1, n_part=2, max_tokens=8, dtype="f32")
    dev = {k: to_dev(v) for k, v in t.items()}
    bad = t["perm"].copy()
    bad[1, 3] = bad[1, 4]  # a neuron named twice
    with pytest.raises(DsmoeError) as ei:
        layer.partition_weights(dev["w1"], dev["w3"], dev["w2"], perm=to_dev(bad))
    assert ei.value.status == -2
    bad2 = t["perm"].copy()
    bad2[0, 0] = 16  # out of range
    with pytest.raises(DsmoeError) as ei:
        layer.partition_weights(dev["w1"], dev["w3"], dev["w2"], perm=to_dev(bad2))
    assert ei.value.status == -2
    layer.partition_weights(dev["w1"], dev["w3"], dev["w2"], perm=dev["perm"])  # the good one passes
    with pytest.raises(DsmoeError):  # T > max_tokens
        layer.forward(torch.zeros((9, 16), device="cuda:0"), torch.zeros((9, 2), device="cuda:0"),
                      torch.zeros((2, 2), device="cuda:0"))
    layer.close()


def test_forward_is_repeatable_and_workspace_reusable(oracle):
    """Two calls with different T and tau on the same context: the second must not see the first."""
    import torch
    spec = spec_of(T=600, D=128, F=256, E=4, K=2, P=2, seed=22)
    t = make_layer(spec)
    layer, dev = make_gpu_layer(spec, t)
    tau_a = tau_table(spec, 0.0)
    r0 = oracle.route(t["logits"], spec.K, spec.P, tau_a)
    tau_b = tau_table(spec, pick_tau(r0.n, spec.P, 0.4))
    ya1 = layer.forward(dev["x"], dev["logits"], to_dev(tau_a)).clone()
    yb = layer.forward(dev["x"][:257].contiguous(), dev["logits"][:257].contiguous(), to_dev(tau_b)).clone()
    ya2 = layer.forward(dev["x"], dev["logits"], to_dev(tau_a)).clone()
    torch.cuda.synchronize()
    assert torch.equal(ya1, ya2)
    sub = {k: (v[:257] if k in ("x", "logits") else v) for k, v in t.items()}
    y_ref = oracle_forward(oracle, spec.with_(T=257), sub, tau_b)
    assert_output_close(to_host64(yb, "bf16"), y_ref, "bf16")
    layer.close()


# ------------------------------------------------------------------ decode-sized batches: split K
SPLIT_CASES = [
    # name, spec, tau, expected number of K ranges GEMM-2 is split into
    ("decode_16_tokens", spec_of(T=16, D=512, F=1024, E=8, K=2, P=4, seed=40), "rate0.25", 8),
    ("uneven_ranges", spec_of(T=40, D=256, F=448, E=4, K=2, P=2, seed=41), "rate0.25", 4),          # 7 stages per part
    ("shared_limits_the_split", spec_of(T=24, D=128, F=512, E=4, K=2, P=2, n_shared=1, F_sh=64, seed=42), "rate0.25", 2),
    ("one_token_split", spec_of(T=1, D=256, F=2048, E=8, K=2, P=2, seed=43), 0.0, 8),
    ("too_many_tiles_to_split", spec_of(T=1200, D=768, F=128, E=64, K=8, P=2, seed=44), "rate0.25", 1),
    # 4 x 17 row tiles (the last of each some 150 rows: no tall items) x 4 column tiles = 272 items of 64 K stages:
    # the few items of the second round are split
    ("last_round_nearly_empty", spec_of(T=8500, D=1024, F=2048, E=4, K=2, P=2, seed=45), 0.0, ">1"),
    # 4 x 16 row tiles + a few rows each, which the last full tiles take along: 256 items, one round, no split
    ("short_last_tiles_leave_one_round", spec_of(T=8200, D=1024, F=2048, E=4, K=2, P=2, seed=45), 0.0, 1),
    # items of 8 K stages: a piece would be all fill and write-out, nothing is split
    ("short_items_stay_whole", spec_of(T=8200, D=1024, F=256, E=4, K=2, P=2, seed=45), 0.0, 1),
    # same with shared experts, whose short contraction (2 stages) limits the split
    ("last_round_with_shared", spec_of(T=5600, D=1024, F=2048, E=4, K=2, P=2, n_shared=1, F_sh=64, seed=46), 0.0, 2),
    ("last_round_under_drop", spec_of(T=8200, D=1024, F=2048, E=4, K=2, P=2, seed=45), "rate0.25", None),
    # a last round at three quarters of the units (192 of 256 items): four pieces each make three full turns of a quarter
    ("last_round_three_quarters_full", spec_of(T=7000, D=2048, F=2048, E=8, K=2, P=2, seed=47), 0.0, None),
]


@pytest.mark.parametrize("name,spec,tau_kind,nsplit", SPLIT_CASES, ids=[c[0] for c in SPLIT_CASES])
def test_gemm2_split_k_on_few_row_tiles(oracle, name, spec, tau_kind, nsplit):
    """With few row tiles the second GEMM splits its contraction into ranges that write partial
    outputs, added in a fixed order by the combine kernel: same result as the oracle, and the
    split only happens while the items stay within one per compute unit."""
    y, y_ref, r, plan = run_case(oracle, spec, tau_kind, expect_mfma=True)
    counters = plan["counters"].cpu().numpy()
    tiles_x_cols = counters[2] * ((spec.D + 255) // 256)
    if nsplit == ">1":
        assert counters[3] > 1, counters
        nsplit = int(counters[3])
    if nsplit is None:  # whatever the plan decided, it must be consistent
        nsplit = int(counters[3])
    assert counters[3] == nsplit, counters
    if tiles_x_cols <= 128:  # every item is split
        assert counters[1] == tiles_x_cols * nsplit and counters[1] <= 256
    elif nsplit > 1:         # only the items of the last round are
        rest = tiles_x_cols % 256
        assert counters[1] == tiles_x_cols + rest * (nsplit - 1) and rest * (nsplit - 1) <= 768
    else:
        assert counters[1] == tiles_x_cols


# ------------------------------------------------- decode-sized batches: GEMM-1 items cut into halves
HALF_CASES = [
    # name, spec, tau, whether the last round of items is expected to get two slots per item
    # 8 experts x 4 parts x 9 neuron tiles = 288 items: the 32 of the second round become 64
    ("last_round_halved", spec_of(T=64, D=128, F=4608, E=8, K=2, P=4, seed=50), 0.0, True),
    ("halved_under_drop", spec_of(T=48, D=128, F=4608, E=8, K=2, P=4, seed=51), "rate0.25", None),
    # 288 routed items + the 4 of the shared experts, which sit last in the list and are among those cut
    ("halved_with_shared", spec_of(T=32, D=128, F=4608, E=8, K=2, P=4, n_shared=1, F_sh=512, seed=52), 0.0, True),
    # the shared experts' row tile has more than 128 rows: their items keep one slot and leave one empty
    ("uncut_shared_items", spec_of(T=200, D=128, F=4480, E=32, K=2, P=1, n_shared=1, F_sh=512, seed=56), 0.0, True),
    # 65..128 rows per expert (three and four blocks of 32 rows in the half-tile kernel variant)
    ("halved_100_rows", spec_of(T=200, D=128, F=2304, E=4, K=2, P=2, seed=57), 0.0, True),
    ("halved_85_rows", spec_of(T=170, D=192, F=2304, E=4, K=2, P=2, seed=58), "rate0.25", None),
    ("first_halves_100_rows", spec_of(T=200, D=128, F=384, E=4, K=2, P=2, seed=59), 0.0, True),
    # 448 items: the second round is three quarters full and stays as it is
    ("last_round_too_full", spec_of(T=64, D=128, F=7168, E=8, K=2, P=4, seed=53), 0.0, False),
    # more than half a tile of rows per expert: not the streaming regime
    ("too_many_rows", spec_of(T=300, D=128, F=4608, E=4, K=2, P=4, seed=54), 0.0, False),
    # the last neuron tile of a partition has 64 neurons: it runs as a first half without a second one
    ("half_empty_neuron_tile", spec_of(T=64, D=128, F=768, E=16, K=2, P=4, seed=55), 0.0, True),
]


@pytest.mark.parametrize("name,spec,tau_kind,halved", HALF_CASES, ids=[c[0] for c in HALF_CASES])
def test_gemm1_items_of_a_sparse_last_round_are_halved(oracle, name, spec, tau_kind, halved):
    """At decode sizes every GEMM-1 item only streams its weight tile, so the step lasts as long
    as its last round of 256 items: when that round is at most half full the plan cuts its items
    into halves of 64 neurons (an item of more than 128 rows, or of a last neuron tile of at most
    64 neurons, stays whole).  Same result as the oracle either way; the item count shows the rule."""
    y, y_ref, r, plan = run_case(oracle, spec, tau_kind, expect_mfma=True)
    counters = plan["counters"].cpu().numpy()
    E_res = spec.hi - spec.lo
    streaming = spec.T * spec.K <= E_res * 128
    rows = np.bincount(r.idx.ravel(), minlength=spec.E)[spec.lo:spec.hi]
    if rows.max() > 256 or (spec.n_shared and spec.T > 256):
        assert not halved and not streaming
        return  # several row tiles per expert: the item count is not this simple
    Fp = spec.F // spec.P
    nt1 = (Fp + 127) // 128
    act = r.group_count.reshape(spec.E, spec.P)[spec.lo:spec.hi] > 0  # sub-experts with a kept unit: one row tile each
    # the list in its order (expert, partition, neuron tile), shared experts last: (rows, neurons of the tile)
    items = [(rows[e], min(128, Fp - 128 * jt)) for e in range(E_res) for p in range(spec.P) if act[e, p] for jt in range(nt1)]
    if spec.n_shared:
        F_sh = spec.n_shared * spec.F_sh
        items += [(spec.T, min(128, F_sh - 128 * jt)) for jt in range((F_sh + 127) // 128)]
    whole = len(items)
    rest = whole % 256
    rule = streaming and 0 < rest <= 128
    if halved is not None:
        assert rule == halved, (whole, rest)
    if not rule:
        assert counters[0] == whole, (counters, whole, rest)
    elif tau_kind == 0.0:  # no drop: every row of an expert keeps every partition
        cuts = sum(1 for n, live in items[whole - rest:] if n <= 128 and live > 64)
        assert counters[0] == whole + cuts, (counters, whole, rest, cuts)
    else:
        assert whole <= counters[0] <= whole + rest, (counters, whole, rest)


# ------------------------------------------------- tall items: a full row tile + the expert's short last tile
TALL_CASES = [
    # name, spec, tau.  Rows per expert = T * K / E on average, spread by the random routing
    ("one_tile_and_a_few_rows", spec_of(T=540, D=128, F=512, E=4, K=2, P=2, seed=60), 0.0),       # ~270 rows per expert
    ("up_to_64_extra_rows", spec_of(T=600, D=192, F=512, E=4, K=2, P=2, seed=61), 0.0),            # ~300
    ("several_tiles_then_a_few_rows", spec_of(T=1060, D=128, F=256, E=4, K=2, P=1, seed=62), 0.0),  # ~530
    ("extra_rows_under_drop", spec_of(T=560, D=128, F=1024, E=4, K=2, P=4, seed=63), "rate0.25"),
    ("extra_rows_general_masks", spec_of(T=373, D=128, F=1024, E=4, K=3, P=4, seed=64), "ragged"),
    ("shared_rows_beyond_a_tile", spec_of(T=270, D=128, F=256, E=4, K=2, P=2, n_shared=1, F_sh=256, seed=65), 0.0),
    ("half_full_last_neuron_tile_stays_plain", spec_of(T=540, D=128, F=384, E=4, K=2, P=2, seed=66), 0.0),  # Fp = 192 = 1.5 tiles
]


@pytest.mark.parametrize("name,spec,tau_kind", TALL_CASES, ids=[c[0] for c in TALL_CASES])
def test_tall_items(oracle, name, spec, tau_kind):
    """When an expert's last row tile has at most 64 rows, the GEMM-1 item of the full tile before it computes
    them too (for every partition whose rows fill that tile) and the short tile gets no item; the GEMM-2 items
    of that tile do the same when the short tile keeps no partition that the full one drops.  Same result as
    the oracle either way; with no drop the item counts show the rule."""
    y, y_ref, r, plan = run_case(oracle, spec, tau_kind, expect_mfma=True, tall_items=1)  # wherever possible: these lists are short
    if tau_kind != 0.0:
        return
    counters = plan["counters"].cpu().numpy()
    Fp = spec.F // spec.P
    nt1 = (Fp + 127) // 128
    tall_ok = Fp % 128 == 0 or Fp % 128 > 64
    if spec.n_shared:
        F_sh = spec.n_shared * spec.F_sh
        tall_ok = tall_ok and (F_sh % 128 == 0 or F_sh % 128 > 64)
    def tiles(n):  # GEMM-1 items per neuron tile for n rows that all keep the partition
        nt = (n + 255) // 256
        return nt - 1 if tall_ok and nt >= 2 and n - (nt - 1) * 256 <= 64 else nt
    rows = np.bincount(r.idx.ravel(), minlength=spec.E)[spec.lo:spec.hi]
    expect = sum(tiles(int(n)) for n in rows) * spec.P * nt1
    merged = sum(1 for n in rows if tiles(int(n)) < (int(n) + 255) // 256)
    if spec.n_shared:
        expect += tiles(spec.T) * ((spec.n_shared * spec.F_sh + 127) // 128)
        merged += tiles(spec.T) < (spec.T + 255) // 256
    if name != "half_full_last_neuron_tile_stays_plain":
        assert merged > 0, rows  # the case is meant to have short last tiles
    else:
        assert merged == 0
    assert counters[0] == expect, (counters, expect, rows)
    tiles2 = sum(tiles(int(n)) for n in rows) + (tiles(spec.T) if spec.n_shared else 0)
    assert counters[2] == tiles2, (counters, tiles2, rows)  # row tiles that have GEMM-2 items


def gemm1_item_counts(spec, r):
    """GEMM-1 items with no drop: (without tall items, with them wherever possible)"""
    nt1 = (spec.F // spec.P + 127) // 128
    rows = np.bincount(r.idx.ravel(), minlength=spec.E)[spec.lo:spec.hi]
    plain = sum((int(n) + 255) // 256 for n in rows) * spec.P * nt1
    merged = sum(1 for n in rows if n > 256 and (int(n) - 1) % 256 < 64)
    return plain, plain - merged * spec.P * nt1


@pytest.mark.parametrize("name,spec,tall_items,expect_tall", [
    # ~270 rows per expert, 8 neuron tiles x 4 partitions: 512 items in two rounds of 256, or 256 tall ones in one
    ("fewer_rounds_pay", spec_of(T=1080, D=128, F=4096, E=8, K=2, P=4, seed=67), 0, True),
    # the same experts with one neuron tile per partition: either list fits one round, and the plain items are the shorter ones
    ("one_round_either_way", spec_of(T=1080, D=128, F=512, E=8, K=2, P=4, seed=67), 0, False),
    ("switched_off", spec_of(T=1080, D=128, F=4096, E=8, K=2, P=4, seed=67), -1, False),
], ids=["fewer_rounds_pay", "one_round_either_way", "switched_off"])
def test_tall_items_are_planned_per_batch(oracle, name, spec, tall_items, expect_tall):
    """cfg.tall_items = 0: the plan prices the GEMM-1 list with and without tall items (items x mean length, in
    whole rounds of one item per compute unit) and takes the cheaper one; -1 switches them off.  Same output."""
    y, y_ref, r, plan = run_case(oracle, spec, 0.0, expect_mfma=True, tall_items=tall_items)
    plain, tall = gemm1_item_counts(spec, r)
    assert tall < plain, (plain, tall)  # the case has short last tiles
    assert int(plan["counters"][0]) == (tall if expect_tall else plain), (plan["counters"], plain, tall)


@pytest.mark.parametrize("dtype,T", [("bf16", 16), ("bf16", 300), ("f32", 40)])
def test_shared_experts_with_a_batch_smaller_than_max_tokens(oracle, dtype, T):
    """The routed rows start right after the shared experts' rows of THIS batch: a context sized
    for more tokens than a call carries must give the same result as one sized exactly."""
    import torch
    if dtype == "bf16":
        spec = spec_of(T=T, D=128, F=256, E=8, K=2, P=2, n_shared=2, F_sh=96, seed=46)
    else:
        spec = spec_of(dtype="f32", T=T, D=40, F=48, E=6, K=2, P=2, n_shared=1, F_sh=24, x_std=0.5, w_std=0.1, seed=47)
    t = make_layer(spec)
    tau = resolve_tau(oracle, spec, t, "rate0.25")
    y_ref = oracle_forward(oracle, spec, t, tau)
    layer, dev = make_gpu_layer(spec, t, max_tokens=1024)
    y = layer.forward(dev["x"], dev["logits"], to_dev(tau))
    torch.cuda.synchronize()
    assert_output_close(to_host64(y, spec.dtype), y_ref, spec.dtype)
    plan = layer.plan(spec.T)
    assert plan["shared_rows"] == (T + plan["tile_rows"] - 1) // plan["tile_rows"] * plan["tile_rows"]
    # importance profiling shares the row layout
    imp = layer.profile_importance(dev["x"], dev["logits"], 1)
    torch.cuda.synchronize()
    assert torch.isfinite(imp).all()
    layer.close()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_one_context_serves_batches_of_different_sizes(oracle, dtype):
    """A serving loop reuses one context and one workspace for batches of any size up to
    max_tokens, large after small and small after large, with different thresholds: nothing a call
    leaves in the workspace may leak into the next."""
    import torch
    if dtype == "bf16":
        spec = spec_of(T=1400, D=128, F=256, E=8, K=2, P=2, n_shared=1, F_sh=64, seed=48)
    else:
        spec = spec_of(dtype="f32", T=300, D=40, F=48, E=6, K=3, P=3, x_std=0.5, w_std=0.1, seed=49)
    t = make_layer(spec)
    layer, dev = make_gpu_layer(spec, t)
    for T, kind in ((spec.T, "rate0.25"), (1, 0.0), (spec.T // 3, "rate0.5"), (17, 2.0), (spec.T, 0.0), (64, "rate0.25")):
        sub = spec.with_(T=T)
        ts = dict(t)
        ts["x"], ts["logits"] = t["x"][:T], t["logits"][:T]
        tau = resolve_tau(oracle, sub, ts, kind)
        y_ref = oracle_forward(oracle, sub, ts, tau)
        y = layer.forward(dev["x"][:T].contiguous(), dev["logits"][:T].contiguous(), to_dev(tau))
        torch.cuda.synchronize()
        assert_output_close(to_host64(y, dtype), y_ref, dtype)
    layer.close()


def test_forward_can_be_captured_in_a_hip_graph_and_replayed(oracle):
    """The forward call only enqueues kernels on the caller's stream (no allocation, no memset, no
    synchronisation), so a serving loop can capture it once and replay it on new inputs placed in
    the same buffers.  Every replay is checked against the eager result and the oracle, with eager
    work and synchronisations between the replays."""
    import torch
    import paper_2508_18376_amd as ds
    spec = spec_of(T=96, D=128, F=256, E=8, K=2, P=2, n_shared=1, F_sh=64, seed=50)
    t = make_layer(spec)
    layer, dev = make_gpu_layer(spec, t)
    x_buf, lg_buf = dev["x"].clone(), dev["logits"].clone()
    tau = resolve_tau(oracle, spec, t, "rate0.25")
    tau_dev = to_dev(tau)
    y_buf = torch.empty((spec.T, spec.D), dtype=torch.bfloat16, device=x_buf.device)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):  # warm-up outside the capture (one-time kernel attributes)
        ds.moe_dualsparse_forward(layer.ctx, layer.packed, x_buf, lg_buf, tau_dev, spec.T, y_buf, layer.workspace, stream)
    stream.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        ds.moe_dualsparse_forward(layer.ctx, layer.packed, x_buf, lg_buf, tau_dev, spec.T, y_buf, layer.workspace,
                                  torch.cuda.current_stream())
    for rep in range(3):
        sub = spec.with_(seed=spec.seed + 10 * rep)
        t2 = make_layer(sub, weights=False)
        x_buf.copy_(to_dev(t2["x"]))
        lg_buf.copy_(to_dev(t2["logits"]))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        y_graph = y_buf.clone()
        y_eager = layer.forward(x_buf, lg_buf, tau_dev)  # eager work between replays
        torch.cuda.synchronize()
        assert torch.equal(y_graph, y_eager)
        ts = dict(t)
        ts["x"], ts["logits"] = t2["x"], t2["logits"]
        r = oracle.route(t2["logits"], spec.K, spec.P, tau)
        if r.min_margin > GUARD:  # thresholds were picked for the first batch; later batches only where safe
            assert_output_close(to_host64(y_graph, "bf16"), oracle_forward(oracle, spec, ts, tau), "bf16")
    layer.close()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_empty_batch_is_a_no_op_everywhere(dtype):
    """T = 0: every entry point returns OK without touching its outputs."""
    import torch
    import paper_2508_18376_amd as ds
    spec = spec_of(dtype=dtype, T=8, D=64, F=64, E=4, K=2, P=2, seed=51)
    t = make_layer(spec)
    layer, dev = make_gpu_layer(spec, t)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    x0 = torch.empty((0, spec.D), dtype=tdt, device="cuda")
    l0 = torch.empty((0, spec.E), dtype=torch.float32, device="cuda")
    tau = to_dev(tau_table(spec, 0.1))
    y = layer.forward(x0, l0, tau)
    assert y.shape == (0, spec.D)
    idx, w, keep, gc = layer.route_and_mask(l0, tau)
    torch.cuda.synchronize()
    assert gc.cpu().numpy().tolist() == [0] * (spec.E * spec.P)
    imp = layer.profile_importance(x0, l0, 0)
    torch.cuda.synchronize()
    assert torch.count_nonzero(imp).item() == 0
    layer.pack_router(to_dev(__import__("synth").make_router(spec)))
    assert layer.router_logits(x0).shape == (0, spec.E)
    assert layer.forward_routed(x0, tau).shape == (0, spec.D)
    # and the context still works afterwards
    y = layer.forward(dev["x"], dev["logits"], tau)
    torch.cuda.synchronize()
    assert torch.isfinite(y.float()).all()
    layer.close()
