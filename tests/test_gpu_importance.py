"""GPU parity of neuron-importance profiling and of the reconstruction order (paper Sec. 4.2 b):
moe_profile_importance against the oracle's accumulated metrics, moe_importance_to_perm against
the plain (importance descending, id ascending) order, and the full chain profile -> perm ->
partition -> forward against the oracle run with the same perm."""
import numpy as np
import pytest

from synth import LayerSpec, make_layer
from gpu_util import make_gpu_layer, to_dev, to_host64, tau_table, assert_output_close, pick_tau

pytestmark = pytest.mark.gpu


def spec_of(**kw):
    base = dict(name="imp", T=700, D=128, F=256, E=4, K=2, P=2, dtype="bf16", seed=31, x_std=1.0, w_std=0.05,
                perm_kind="identity")
    base.update(kw)
    return LayerSpec(**base)


CASES = [
    ("bf16_mfma", spec_of()),
    ("bf16_fine", spec_of(T=900, D=64, F=128, E=16, K=4, seed=32)),
    ("bf16_window", spec_of(T=600, E=8, resident=(2, 5), seed=33)),
    ("f32_generic", spec_of(dtype="f32", T=150, D=40, F=72, E=5, K=2, P=3, seed=34)),
    ("empty_expert", spec_of(T=3, E=16, K=2, seed=35)),
    # 8 x 4 x 9 = 288 GEMM-1 items at a decode-sized batch: the items of the last round are cut into halves
    ("halved_items", spec_of(T=64, D=128, F=4608, E=8, K=2, P=4, seed=37)),
]


@pytest.mark.parametrize("name,spec", CASES, ids=[c[0] for c in CASES])
@pytest.mark.parametrize("metric", [0, 1, 2, 3])
def test_importance_matches_oracle(oracle, name, spec, metric):
    import torch
    t = make_layer(spec)
    imp_ref, abs_ref = oracle.importance(t["x"], t["logits"], t["w1"], t["w3"], spec.K, metric, lo=spec.lo, hi=spec.hi)
    tt = dict(t)
    tt["perm"] = None  # profiling runs on weights packed in their original neuron order
    layer, dev = make_gpu_layer(spec, tt)
    imp = layer.profile_importance(dev["x"], dev["logits"], metric)
    torch.cuda.synchronize()
    got = imp.cpu().numpy().astype(np.float64)
    # fp32 terms (fp32 accumulation of exact products, then Swish) summed in fp32 in a fixed order on
    # both paths: the error is a few fp32 roundings per term, bounded against the sum of |terms|
    assert np.all(np.abs(got - imp_ref) <= IMP_TOL * abs_ref + 1e-6 * max(abs_ref.max(), 1e-30))
    if spec.T * spec.K >= 100 * spec.E:  # sums over a hundred rows and more: single terms that cancel no longer set the scale
        assert np.all(np.abs(got - imp_ref) <= IMP_TOL_SUMS * abs_ref)
    layer.close()


IMP_TOL = 3e-5       # relative to the sum of the |terms| of a neuron (a lone term can lose that much to cancellation in x W1)
IMP_TOL_SUMS = 2e-6  # the same for sums over many rows (measured: 1e-7 .. 4e-7)


@pytest.mark.parametrize("metric", [1, 3])
def test_gpu_order_equals_the_oracle_order_on_separated_importances(oracle, metric):
    """Calibration tokens -> importance -> order, all on the GPU, against the oracle's order: equal
    wherever the oracle's adjacent importances lie farther apart than the GPU's error bound (a seed
    is searched whose every gap does)."""
    import torch
    for seed in range(40, 80):
        spec = spec_of(T=500, D=64, F=96, E=3, K=2, P=2, seed=seed)
        t = make_layer(spec)
        imp_ref, abs_ref = oracle.importance(t["x"], t["logits"], t["w1"], t["w3"], spec.K, metric)
        srt = -np.sort(-imp_ref, axis=1)
        if np.all(srt[:, :-1] - srt[:, 1:] > 4 * IMP_TOL_SUMS * abs_ref.max()):
            break
    else:
        pytest.skip("no seed with well separated importances")
    tt = dict(t)
    tt["perm"] = None
    layer, dev = make_gpu_layer(spec, tt)
    perm = layer.importance_to_perm(layer.profile_importance(dev["x"], dev["logits"], metric))
    torch.cuda.synchronize()
    np.testing.assert_array_equal(perm.cpu().numpy(), oracle.perm_from_importance(imp_ref))
    layer.close()


def test_importance_is_independent_of_the_activation_scale_setting(oracle):
    """cfg.h_scale_log2 rescales the packed up projection; the profiled importance must not change."""
    import torch
    spec = spec_of(T=400, seed=38)
    t = make_layer(spec)
    tt = dict(t)
    tt["perm"] = None
    ref = None
    for k in (0, 5, -3):
        layer, dev = make_gpu_layer(spec, tt, h_scale_log2=k)
        got = [layer.profile_importance(dev["x"], dev["logits"], m).cpu().numpy() for m in range(4)]
        torch.cuda.synchronize()
        if ref is None:
            ref = got
        else:
            for a, b in zip(got, ref):  # powers of two: the same terms; the order of the rows inside a tile may differ from run to run
                np.testing.assert_allclose(a, b, rtol=2e-6, atol=2e-6 * np.abs(b).max())
        layer.close()


def test_perm_from_importance_is_the_plain_order(oracle):
    import torch
    from paper_2508_18376_amd import DualSparseLayer
    rng = np.random.default_rng(3)
    E, F = 3, 2500  # spans several 1024-value tiles of the rank kernel
    imp = rng.standard_normal((E, F)).astype(np.float32)
    imp[0, ::7] = 0.25          # many exact ties
    imp[1] = 1.0                # all equal: identity order
    layer = DualSparseLayer(d_model=32, d_ff=F, n_experts=E, top_k=1, n_part=1, max_tokens=8, dtype="f32")
    perm = layer.importance_to_perm(to_dev(imp))
    torch.cuda.synchronize()
    np.testing.assert_array_equal(perm.cpu().numpy(), oracle.perm_from_importance(imp.astype(np.float64)))
    assert list(perm[1].cpu().numpy()) == list(range(F))
    layer.close()


def test_perm_from_importance_with_nan_is_still_a_permutation():
    import torch
    from paper_2508_18376_amd import DualSparseLayer
    rng = np.random.default_rng(5)
    E, F = 2, 1500
    imp = rng.standard_normal((E, F)).astype(np.float32)
    bad = rng.choice(F, size=40, replace=False)
    imp[0, bad] = np.nan
    imp[1, :] = np.nan
    layer = DualSparseLayer(d_model=32, d_ff=F, n_experts=E, top_k=1, n_part=1, max_tokens=8, dtype="f32")
    perm = layer.importance_to_perm(to_dev(imp)).cpu().numpy()
    torch.cuda.synchronize()
    for e in range(E):
        assert sorted(perm[e]) == list(range(F))
    assert list(perm[0][-40:]) == sorted(bad.tolist())            # NaN neurons last, by id
    v = imp[0][perm[0][:-40]]
    assert np.all(v[:-1] >= v[1:])
    assert list(perm[1]) == list(range(F))
    layer.close()


def test_profile_then_partition_then_forward(oracle):
    """Reconstruction end to end: importance (metric 1) -> perm -> packed weights -> dual-threshold
    forward; the oracle runs the layer with the permutation the GPU produced."""
    import torch
    spec = spec_of(T=800, D=128, F=256, E=4, K=2, P=2, seed=36)
    t = make_layer(spec)
    tt = dict(t)
    tt["perm"] = None
    layer, dev = make_gpu_layer(spec, tt)
    imp = layer.profile_importance(dev["x"], dev["logits"], 1)
    perm = layer.importance_to_perm(imp)
    torch.cuda.synchronize()
    perm_h = perm.cpu().numpy()
    imp_h = imp.cpu().numpy()
    for e in range(spec.E):  # a valid permutation, ordered by the GPU's own importance values
        assert sorted(perm_h[e]) == list(range(spec.F))
        v = imp_h[e][perm_h[e]]
        assert np.all(v[:-1] >= v[1:])
    layer.partition_weights(dev["w1"], dev["w3"], dev["w2"], perm=perm)
    r0 = oracle.route(t["logits"], spec.K, spec.P, np.zeros((spec.E, spec.P), np.float32))
    tau = tau_table(spec, pick_tau(r0.n, spec.P, 0.3))
    y = layer.forward(dev["x"], dev["logits"], to_dev(tau))
    torch.cuda.synchronize()
    y_ref = oracle.forward(t["x"], t["logits"], t["w1"], t["w3"], t["w2"], tau, spec.K, spec.P, perm=perm_h)
    assert_output_close(to_host64(y, "bf16"), y_ref, "bf16")
    layer.close()
