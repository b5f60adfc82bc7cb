"""GPU parity of the gating product l = x W_g, of the layer driven by its own router
(moe_dualsparse_forward_routed) and of the complete transformation (paper Sec. 3.1)."""
import numpy as np
import pytest

from synth import LayerSpec, make_layer, make_router
from gpu_util import make_gpu_layer, to_dev, to_host64, tau_table, pick_tau, assert_output_close

pytestmark = pytest.mark.gpu

# fp32 accumulation of exact products in an order that differs from the oracle's: at most ~80
# roundings lie on the path of any product (64-step partial sums, four-way and tree reductions)
LOGIT_TOL = 80 * 2.0 ** -24
# routing decisions are compared only where the oracle's margin is far above the logit error
LOGIT_MARGIN = 1e-4
SCORE_MARGIN = 2e-5


def spec_of(**kw):
    base = dict(name="rt", T=300, D=128, F=128, E=8, K=2, P=2, dtype="bf16", seed=51, x_std=1.0, w_std=0.05)
    base.update(kw)
    return LayerSpec(**base)


def widen(a):
    from synth import bf16_bits_to_f32
    return bf16_bits_to_f32(a).astype(np.float64) if a.dtype == np.uint16 else a.astype(np.float64)


def check_logits(got, x, wg, oracle):
    ref = oracle.router_logits(x, wg)
    bound = LOGIT_TOL * np.matmul(np.abs(widen(x)), np.abs(widen(wg))) + 1e-30
    assert got.shape == ref.shape
    assert np.all(np.abs(got.astype(np.float64) - ref) <= bound), float((np.abs(got - ref) / bound).max())
    return ref


ROUTER_CASES = [
    ("bf16_E8", spec_of()),
    ("bf16_E64_ragged_T", spec_of(T=70, D=256, E=64, K=8)),
    ("bf16_three_steps", spec_of(T=33, D=192, E=40, K=4)),
    ("bf16_E160_two_groups", spec_of(T=97, D=128, E=160, K=6)),
    ("bf16_one_token", spec_of(T=1, D=64, E=8)),
    ("bf16_generic_D96", spec_of(T=50, D=96, E=12, K=3)),
    ("f32_generic", spec_of(T=45, D=40, E=5, K=2, dtype="f32")),
]


@pytest.mark.parametrize("name,spec", ROUTER_CASES, ids=[c[0] for c in ROUTER_CASES])
def test_router_logits_match_the_oracle(oracle, name, spec):
    import torch
    from paper_2508_18376_amd import DualSparseLayer
    t = make_layer(spec, weights=False)
    wg = make_router(spec)
    layer = DualSparseLayer(d_model=spec.D, d_ff=spec.F, n_experts=spec.E, top_k=spec.K, n_part=spec.P,
                            max_tokens=spec.T, dtype=spec.dtype)
    layer.pack_router(to_dev(wg))
    got = layer.router_logits(to_dev(t["x"]))
    torch.cuda.synchronize()
    check_logits(got.cpu().numpy(), t["x"], wg, oracle)
    layer.close()


def safe_routing_inputs(oracle, spec, rate):
    """Seeds are advanced until every token's Top-K cut and every kept/dropped decision of the
    oracle has a margin far above the error of the GPU's logits."""
    for s in range(spec.seed, spec.seed + 40):
        sp = spec.with_(seed=s)
        t = make_layer(sp)
        wg = make_router(sp)
        logits = oracle.router_logits(t["x"], wg).astype(np.float32)
        srt = np.sort(logits, axis=1)[:, ::-1]
        if sp.K < sp.E and (srt[:, sp.K - 1] - srt[:, sp.K]).min() < LOGIT_MARGIN:
            continue
        if sp.K > 1 and np.diff(srt[:, :sp.K], axis=1).max() > -LOGIT_MARGIN:  # order inside the selection
            continue
        r0 = oracle.route(logits, sp.K, sp.P, np.zeros((sp.E, sp.P), np.float32), lo=sp.lo, hi=sp.hi)
        tau = tau_table(sp, pick_tau(r0.n, sp.P, rate))
        if rate > 0 and oracle.route(logits, sp.K, sp.P, tau, lo=sp.lo, hi=sp.hi).min_margin < SCORE_MARGIN:
            continue
        return sp, t, wg, logits, tau
    raise AssertionError("no seed with safe routing margins")


ROUTED_CASES = [
    ("bf16_mfma_drop30", spec_of(T=500, D=128, F=256, E=8, K=2, P=2), 0.3),
    ("bf16_mfma_no_drop", spec_of(T=300, D=128, F=128, E=8, K=2, P=2), 0.0),
    ("bf16_fine_grained", spec_of(T=260, D=256, F=64, E=32, K=4, P=2, seed=60), 0.25),
    ("f32_generic", spec_of(T=120, D=40, F=36, E=5, K=2, P=3, dtype="f32", seed=70), 0.3),
]


@pytest.mark.parametrize("name,spec,rate", ROUTED_CASES, ids=[c[0] for c in ROUTED_CASES])
def test_layer_driven_by_its_own_router(oracle, name, spec, rate):
    import torch
    sp, t, wg, logits, tau = safe_routing_inputs(oracle, spec, rate)
    layer, dev = make_gpu_layer(sp, {k: v for k, v in t.items() if k != "logits"})
    layer.pack_router(to_dev(wg))
    y, lg = layer.forward_routed(dev["x"], to_dev(tau), want_logits=True)
    torch.cuda.synchronize()
    check_logits(lg.cpu().numpy(), t["x"], wg, oracle)
    plan = layer.plan(sp.T)
    r = oracle.route(logits, sp.K, sp.P, tau, lo=sp.lo, hi=sp.hi)
    np.testing.assert_array_equal(plan["topk_idx"].cpu().numpy().reshape(sp.T, sp.K), r.idx)
    np.testing.assert_array_equal(plan["keep_bits"].cpu().numpy().reshape(sp.T, sp.K), r.keep_bits)
    y_ref = oracle.forward(t["x"], logits, t["w1"], t["w3"], t["w2"], tau, sp.K, sp.P, perm=t["perm"], lo=sp.lo, hi=sp.hi)
    assert_output_close(to_host64(y, sp.dtype), y_ref, sp.dtype)
    # logits kept in the workspace: same output
    y2 = layer.forward_routed(dev["x"], to_dev(tau))
    torch.cuda.synchronize()
    assert torch.equal(y, y2)
    layer.close()


TRANSFORM_CASES = [
    ("f32_P2_perm", spec_of(T=4, D=24, F=36, E=4, P=2, dtype="f32"), True),
    ("f32_P3_rounded_scale", spec_of(T=4, D=10, F=30, E=3, P=3, dtype="f32"), True),
    ("bf16_P4_perm", spec_of(T=4, D=64, F=512, E=4, P=4), True),
    ("bf16_P3_rounded_scale", spec_of(T=4, D=32, F=96, E=2, P=3), True),
    ("bf16_identity_order", spec_of(T=4, D=32, F=64, E=4, P=2), False),
    ("bf16_window", spec_of(T=4, D=32, F=64, E=8, P=2, resident=(2, 5)), True),
]


@pytest.mark.parametrize("name,spec,use_perm", TRANSFORM_CASES, ids=[c[0] for c in TRANSFORM_CASES])
def test_complete_transformation_is_bit_exact(oracle, name, spec, use_perm):
    import torch
    from paper_2508_18376_amd import DualSparseLayer
    t = make_layer(spec)
    wg = make_router(spec)
    perm = t["perm"] if use_perm else None
    want = oracle.complete_transform(wg[:, spec.lo:spec.hi], t["w1"], t["w3"], t["w2"], spec.P, perm=perm)
    wg_want = np.repeat(wg, spec.P, axis=1)  # the router keeps all E columns
    layer = DualSparseLayer(d_model=spec.D, d_ff=spec.F, n_experts=spec.E, top_k=spec.K, n_part=spec.P, max_tokens=8,
                            dtype=spec.dtype, expert_lo=spec.lo, expert_hi=spec.hi)
    got = layer.transform_complete(to_dev(wg), to_dev(t["w1"]), to_dev(t["w3"]), to_dev(t["w2"]), perm=to_dev(perm))
    torch.cuda.synchronize()

    def bits(tensor):
        return tensor.view(torch.int16).cpu().numpy().view(np.uint16) if tensor.dtype == torch.bfloat16 else tensor.cpu().numpy()

    np.testing.assert_array_equal(bits(got[0]), wg_want)
    np.testing.assert_array_equal(bits(got[0])[:, spec.lo * spec.P:spec.hi * spec.P], want[0])
    for g, w in zip(got[1:], want[1:]):
        np.testing.assert_array_equal(bits(g), w)
    layer.close()


def test_transform_rejects_a_non_permutation():
    import torch
    from paper_2508_18376_amd import DualSparseLayer, DsmoeError
    spec = spec_of(T=4, D=32, F=64, E=2, P=2)
    t = make_layer(spec)
    bad = t["perm"].copy()
    bad[1, 5] = bad[1, 6]
    layer = DualSparseLayer(d_model=spec.D, d_ff=spec.F, n_experts=spec.E, top_k=spec.K, n_part=spec.P, max_tokens=8)
    with pytest.raises(DsmoeError) as ei:
        layer.transform_complete(None, to_dev(t["w1"]), to_dev(t["w3"]), to_dev(t["w2"]), perm=to_dev(bad))
    assert ei.value.status == -2
    layer.close()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_transformed_layer_runs_as_a_plain_layer_and_reproduces_the_original(oracle, dtype):
    """Sec. 3.1 end to end on the GPU: transform -> a second context with E*P experts, Top-(K*P),
    one part per expert -> same output as the oracle's ORIGINAL layer; with thresholds tau / P it
    drops like the original layer under the single threshold tau."""
    import torch
    from paper_2508_18376_amd import DualSparseLayer
    P = 2
    base = spec_of(T=400, D=128, F=256, E=8, K=2, P=P, dtype=dtype, seed=80) if dtype == "bf16" else \
        spec_of(T=150, D=48, F=40, E=6, K=2, P=P, dtype=dtype, seed=81)
    sp, t, wg, logits, _ = safe_routing_inputs(oracle, base, 0.0)
    first = DualSparseLayer(d_model=sp.D, d_ff=sp.F, n_experts=sp.E, top_k=sp.K, n_part=P, max_tokens=sp.T, dtype=dtype)
    wg_t, w1_t, w3_t, w2_t = first.transform_complete(to_dev(wg), to_dev(t["w1"]), to_dev(t["w3"]), to_dev(t["w2"]),
                                                      perm=to_dev(t["perm"]))
    first.close()
    second = DualSparseLayer(d_model=sp.D, d_ff=sp.F // P, n_experts=sp.E * P, top_k=sp.K * P, n_part=1, max_tokens=sp.T,
                             dtype=dtype)
    second.partition_weights(w1_t, w3_t, w2_t)
    second.pack_router(wg_t)
    x = to_dev(t["x"])
    # no drop: the original layer's output
    y = second.forward_routed(x, to_dev(np.zeros((sp.E * P, 1), np.float32)))
    torch.cuda.synchronize()
    tau0 = np.zeros((sp.E, P), np.float32)
    y_ref = oracle.forward(t["x"], logits, t["w1"], t["w3"], t["w2"], tau0, sp.K, P, perm=t["perm"])
    assert_output_close(to_host64(y, dtype), y_ref, dtype)
    # single threshold tau on the original layer <-> tau / P on the transformed one
    r0 = oracle.route(logits, sp.K, P, tau0)
    tau = float(pick_tau(r0.n, 1, 0.3)[0])
    rt = oracle.route(np.repeat(logits, P, axis=1), sp.K * P, 1, np.full((sp.E * P, 1), tau / P, np.float32))
    ro = oracle.route(logits, sp.K, P, np.full((sp.E, P), tau, np.float32))
    assert min(rt.min_margin * P, ro.min_margin) > SCORE_MARGIN
    y = second.forward_routed(x, to_dev(np.full((sp.E * P, 1), tau / P, np.float32)))
    torch.cuda.synchronize()
    y_ref = oracle.forward(t["x"], logits, t["w1"], t["w3"], t["w2"], np.full((sp.E, P), tau, np.float32), sp.K, P,
                           perm=t["perm"])
    assert np.abs(y_ref).max() > 0
    assert_output_close(to_host64(y, dtype), y_ref, dtype)
    second.close()
