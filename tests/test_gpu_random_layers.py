"""Seeded random layer configurations against the oracle: shapes, expert counts, partitions,
shared experts, resident windows, batch sizes below max_tokens and threshold tables are all drawn
at random inside the limits of the configuration (one list, fixed by the seeds below)."""
import numpy as np
import pytest

from synth import LayerSpec, make_layer
from plan_cover import check_cover
from gpu_util import GUARD, make_gpu_layer, to_dev, to_host64, pick_tau, tau_table, assert_output_close

pytestmark = pytest.mark.gpu


def draw_case(seed):
    rng = np.random.default_rng(1000 + seed)
    kind = ["bf16_mfma", "bf16_mfma", "bf16_generic", "f32"][seed % 4]
    E = int(rng.choice([1, 2, 3, 8, 8, 16, 33, 64, 70]))
    K = int(rng.integers(1, min(E, 8) + 1))
    P = int(rng.choice([1, 2, 2, 3, 4, 8]))
    if kind == "bf16_mfma":
        D = 32 * int(rng.integers(1, 11))
        Fp = 32 * int(rng.integers(1, 6))
        F_sh = 32 * int(rng.integers(1, 4))
    else:
        D = int(rng.integers(5, 90))
        Fp = int(rng.integers(3, 50))
        F_sh = int(rng.integers(3, 40))
    n_shared = int(rng.choice([0, 0, 1, 2]))
    T = int(rng.choice([1, 2, 17, 64, 65, 200, 333, 700]))
    max_tokens = T + int(rng.choice([0, 1, 300]))
    lo = int(rng.integers(0, E)) if E > 1 and rng.random() < 0.4 else 0
    hi = int(rng.integers(lo + 1, E + 1)) if lo > 0 or (E > 1 and rng.random() < 0.3) else E
    tau_kind = ["zero", "rate", "ragged", "rate", "ragged", "rate", "ragged", "all"][int(rng.integers(0, 8))]
    spec = LayerSpec(name="rnd%d" % seed, T=T, D=D, F=Fp * P, E=E, K=K, P=P, dtype="f32" if kind == "f32" else "bf16",
                     seed=2000 + seed, n_shared=n_shared, F_sh=F_sh if n_shared else 0, resident=(lo, hi),
                     x_std=1.0, w_std=float(rng.choice([0.05, 0.2])), perm_kind=str(rng.choice(["random", "identity", "reversed"])))
    return spec, max_tokens, tau_kind, bool(rng.random() < 0.3), kind


def draw_medium_case(seed):
    """Matrix-core path only, several row tiles per expert: full tiles, ragged tails of every length, half
    neuron tiles, K splits of short item lists, all at once."""
    rng = np.random.default_rng(5000 + seed)
    E = int(rng.choice([1, 2, 4, 8, 16]))
    K = int(rng.integers(1, min(E, 4) + 1))
    P = int(rng.choice([1, 2, 2, 4, 4, 8]))
    D = 32 * int(rng.integers(2, 25))
    Fp = 32 * int(rng.integers(1, 13))
    F_sh = 32 * int(rng.integers(1, 9))
    n_shared = int(rng.choice([0, 0, 1, 2]))
    T = int(rng.integers(200, 3000))
    max_tokens = T + int(rng.choice([0, 1, 500]))
    lo = int(rng.integers(0, E)) if E > 1 and rng.random() < 0.3 else 0
    hi = int(rng.integers(lo + 1, E + 1)) if lo > 0 or (E > 1 and rng.random() < 0.2) else E
    tau_kind = ["zero", "rate", "ragged", "rate", "ragged", "rate"][int(rng.integers(0, 6))]
    spec = LayerSpec(name="med%d" % seed, T=T, D=D, F=Fp * P, E=E, K=K, P=P, dtype="bf16", seed=7000 + seed, n_shared=n_shared,
                     F_sh=F_sh if n_shared else 0, resident=(lo, hi), x_std=1.0, w_std=float(rng.choice([0.05, 0.2])),
                     perm_kind=str(rng.choice(["random", "identity", "reversed"])))
    return spec, max_tokens, tau_kind, bool(rng.random() < 0.3), "bf16_mfma"


def draw_large_case(seed):
    """Matrix-core path, work lists of many rounds of items (thousands of tokens): where the plan prices
    lists with and without tall items, splits the last round of GEMM-2 and orders items for the XCDs."""
    rng = np.random.default_rng(9000 + seed)
    E = int(rng.choice([4, 8, 16, 32]))
    K = int(rng.integers(1, 5))
    P = int(rng.choice([1, 2, 4]))
    D = 64 * int(rng.integers(2, 9))
    Fp = 128 * int(rng.integers(1, 7)) + int(rng.choice([0, 0, 96]))
    F_sh = 128 * int(rng.integers(1, 5))
    n_shared = int(rng.choice([0, 0, 1]))
    T = int(rng.integers(1500, 7000))
    max_tokens = T + int(rng.choice([0, 300]))
    tau_kind = ["zero", "rate", "rate", "ragged"][int(rng.integers(0, 4))]
    spec = LayerSpec(name="big%d" % seed, T=T, D=D, F=Fp * P, E=E, K=K, P=P, dtype="bf16", seed=9500 + seed, n_shared=n_shared,
                     F_sh=F_sh if n_shared else 0, resident=(0, E), x_std=1.0, w_std=float(rng.choice([0.05, 0.2])),
                     perm_kind=str(rng.choice(["random", "identity"])))
    return spec, max_tokens, tau_kind, bool(rng.random() < 0.3), "bf16_mfma"


CASES = [draw_case(s) for s in range(32)] + [draw_medium_case(s) for s in range(24)] + [draw_large_case(s) for s in range(12)]


@pytest.mark.parametrize("spec,max_tokens,tau_kind,renorm,kind", CASES, ids=["%s_%s" % (c[0].name, c[4]) for c in CASES])
def test_random_layer(oracle, spec, max_tokens, tau_kind, renorm, kind):
    import torch
    t = make_layer(spec)
    zero = np.zeros((spec.E, spec.P), np.float32)
    r0 = oracle.route(t["logits"], spec.K, spec.P, zero, spec.lo, spec.hi)
    if tau_kind == "zero":
        tau = zero
    elif tau_kind == "all":
        tau = np.full((spec.E, spec.P), 2.0, np.float32)
    elif tau_kind == "rate" and spec.K > 1 and r0.n.size >= 8:
        tau = tau_table(spec, pick_tau(r0.n, spec.P, 0.3))
    else:
        tau = zero
        for attempt in range(60):
            cand = np.random.default_rng(spec.seed + 7 * attempt).uniform(0.02, 0.7, (spec.E, spec.P)).astype(np.float32)
            if oracle.route(t["logits"], spec.K, spec.P, cand, spec.lo, spec.hi).min_margin > 2 * GUARD:
                tau = cand
                break
    r = oracle.route(t["logits"], spec.K, spec.P, tau, spec.lo, spec.hi, renorm=renorm)
    if 0 < r.keep.sum() < r.keep.size and spec.K > 1:
        assert r.min_margin > GUARD
    y_ref = oracle.forward(t["x"], t["logits"], t["w1"], t["w3"], t["w2"], tau, spec.K, spec.P, perm=t["perm"],
                           sh_w1=t.get("sh_w1"), sh_w3=t.get("sh_w3"), sh_w2=t.get("sh_w2"), lo=spec.lo, hi=spec.hi,
                           renorm=renorm)
    # tall work items: left to the plan, forced, forbidden, forced (these lists are mostly too short for the plan to want them)
    tall_items = (0, 1, -1, 1)[spec.seed % 4]
    layer, dev = make_gpu_layer(spec, t, max_tokens=max_tokens, renorm=renorm, tall_items=tall_items)
    assert layer.uses_mfma == (kind == "bf16_mfma")
    y = layer.forward(dev["x"], dev["logits"], to_dev(tau))
    torch.cuda.synchronize()
    plan = layer.plan(spec.T)
    np.testing.assert_array_equal(plan["topk_idx"].cpu().numpy(), r.idx)
    np.testing.assert_array_equal(plan["keep_bits"].cpu().numpy(), r.keep_bits)
    assert_output_close(to_host64(y, spec.dtype), y_ref, spec.dtype)
    if kind == "bf16_mfma":  # and the work lists behind that result cover every kept unit exactly once
        check_cover({k: (v.cpu().numpy() if hasattr(v, "cpu") else v) for k, v in plan.items()}, name=spec.name, T=spec.T, D=spec.D,
                    F=spec.F, P=spec.P, E_res=spec.hi - spec.lo, n_shared=spec.n_shared, F_sh=spec.F_sh)
    layer.close()
