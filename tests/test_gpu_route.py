"""GPU parity, routing and masks: moe_route_and_mask against the oracle, bit-exact indices, keep
bits and group counts (ties to the lower index), weights to float rounding.  Every input is
checked to sit outside the guard band |n - tau| > 1e-6 where fp32 and fp64 could disagree."""
import numpy as np
import pytest

from synth import LayerSpec, LAYERS, make_logits
from gpu_util import GUARD, to_dev, pick_tau, tau_table

pytestmark = pytest.mark.gpu



def spec_of(**kw):
    base = dict(name="r", T=777, D=64, F=64, E=8, K=2, P=2, dtype="f32", seed=5)
    base.update(kw)
    return LayerSpec(**base)


CASES = [
    ("C1", LAYERS["C1"], 0.2, False),
    ("E8K2P4", spec_of(T=4096, E=8, K=2, P=4, seed=1), "rate0.25", False),
    ("E64K8", spec_of(T=3000, E=64, K=8, P=2, seed=2), "rate0.25", False),
    ("E64K6renorm", spec_of(T=1001, E=64, K=6, P=2, seed=3), "rate0.33", True),
    ("E16K4P3", spec_of(T=513, F=96, E=16, K=4, P=3, seed=4), "rate0.5", False),
    ("E32K16", spec_of(T=100, E=32, K=16, P=1, seed=6), "rate0.1", False),
    ("E128K4wave", spec_of(T=700, E=128, K=4, P=2, seed=7), "rate0.25", False),
    ("E300K6wave", spec_of(T=300, E=300, K=6, P=8, seed=8), "rate0.25", True),
    ("E512K16wave", spec_of(T=65, E=512, K=16, P=2, seed=9), "rate0.25", False),
    # expert counts that are not multiples of 4 (unaligned logit rows: scalar loads), small and large batches
    ("E50K3rows", spec_of(T=500, E=50, K=3, P=2, seed=13), "rate0.25", False),
    ("E131K5big", spec_of(T=2500, E=131, K=5, P=2, seed=14), "rate0.25", True),
    # more than 2048 tokens: 64 tokens per block, 2 / 4 / 8 chunks of 64 experts per lane row
    ("E128K4big", spec_of(T=2100, E=128, K=4, P=2, seed=15), "rate0.25", False),
    ("E256K8big", spec_of(T=2100, E=256, K=8, P=4, seed=16), "rate0.25", False),
    ("E512K6big", spec_of(T=2050, E=512, K=6, P=2, seed=17), "rate0.33", False),
    ("window", spec_of(T=2000, E=8, K=2, P=4, seed=10, resident=(2, 5)), "rate0.25", False),
    ("zipf", LAYERS["C5"].with_(T=2048), "rate0.25", False),
    ("K1", spec_of(T=64, E=5, K=1, P=2, seed=11), 1.0, False),
    ("E1", spec_of(T=10, E=1, K=1, P=1, seed=12), 0.5, False),
]


@pytest.mark.parametrize("name,spec,tau_kind,renorm", CASES, ids=[c[0] for c in CASES])
def test_route_and_mask_bit_exact(oracle, name, spec, tau_kind, renorm):
    import torch
    from paper_2508_18376_amd import DualSparseLayer
    logits = make_logits(spec)
    if name == "E16K4P3":
        logits[::5] = np.round(logits[::5] * 2) / 2  # exact ties in the logits
    if isinstance(tau_kind, str):
        r0 = oracle.route(logits, spec.K, spec.P, np.zeros((spec.E, spec.P), np.float32), spec.lo, spec.hi)
        tau = tau_table(spec, pick_tau(r0.n, spec.P, float(tau_kind[4:])))
    else:
        tau = tau_table(spec, tau_kind)
    ref = oracle.route(logits, spec.K, spec.P, tau, spec.lo, spec.hi, renorm=renorm)
    if name not in ("K1",):  # K = 1 sits exactly on tau = 1 on purpose (n is exactly 1 on both sides)
        assert ref.min_margin > GUARD, ref.min_margin
    layer = DualSparseLayer(d_model=spec.D, d_ff=spec.F, n_experts=spec.E, top_k=spec.K, n_part=spec.P,
                            max_tokens=spec.T, dtype=spec.dtype, expert_lo=spec.lo, expert_hi=spec.hi,
                            renorm_combine=renorm)
    idx, w, keep, gc = layer.route_and_mask(to_dev(logits), to_dev(tau))
    torch.cuda.synchronize()
    np.testing.assert_array_equal(idx.cpu().numpy(), ref.idx)
    np.testing.assert_array_equal(keep.cpu().numpy(), ref.keep_bits)
    np.testing.assert_array_equal(gc.cpu().numpy().astype(np.int64), ref.group_count)
    np.testing.assert_allclose(w.cpu().numpy().astype(np.float64), ref.g, rtol=2e-6, atol=1e-30)
    layer.close()


def test_route_zero_tokens_and_limits():
    import torch
    from paper_2508_18376_amd import DualSparseLayer, DsmoeError
    layer = DualSparseLayer(d_model=64, d_ff=64, n_experts=8, top_k=2, n_part=2, max_tokens=16, dtype="f32")
    tau = torch.zeros((8, 2), dtype=torch.float32, device="cuda:0")
    idx, w, keep, gc = layer.route_and_mask(torch.zeros((0, 8), dtype=torch.float32, device="cuda:0"), tau)
    torch.cuda.synchronize()
    assert idx.shape == (0, 2) and int(gc.sum()) == 0
    with pytest.raises(DsmoeError):
        layer.route_and_mask(torch.zeros((17, 8), dtype=torch.float32, device="cuda:0"), tau)
    layer.close()


@pytest.mark.parametrize("E,K", [(8, 2), (64, 8), (160, 6)])
def test_non_finite_logits_still_give_valid_expert_ids(E, K):
    """NaN / infinite router logits give unspecified scores but never an invalid selection: K
    distinct expert ids in range per token, and the layer's later steps stay in bounds."""
    import torch
    from paper_2508_18376_amd import DualSparseLayer
    rng = np.random.default_rng(E)
    T = 200
    logits = rng.standard_normal((T, E)).astype(np.float32)
    logits[0, :] = np.nan
    logits[1, :] = -np.inf
    logits[2, ::2] = np.inf
    logits[3, 1] = np.nan
    logits[4:40, rng.integers(0, E, 36)] = np.nan
    layer = DualSparseLayer(d_model=32, d_ff=32, n_experts=E, top_k=K, n_part=1, max_tokens=T, dtype="f32")
    idx, w, keep, gc = layer.route_and_mask(to_dev(logits), to_dev(np.full((E, 1), 0.1, np.float32)))
    torch.cuda.synchronize()
    idx = idx.cpu().numpy()
    assert idx.min() >= 0 and idx.max() < E
    assert all(len(set(row)) == K for row in idx)
    finite = np.isfinite(logits).all(axis=1)
    ref_top = np.argsort(-logits[finite], axis=1, kind="stable")[:, :K]
    np.testing.assert_array_equal(idx[finite], ref_top)
    layer.close()
