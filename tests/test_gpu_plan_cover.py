"""GPU, plan invariants: the work lists that the plan kernel hands to the two grouped GEMMs cover every
kept unit exactly once.  The parity tests cannot see a tile that is computed twice (same result, wasted
time), and see a missing one only through the numbers; here the lists themselves are read back
(dsmoe_plan_layout fields 12 and 13) and checked against the rows' keep patterns:

* first GEMM (Eq. 4 per sub-expert): every row that keeps partition p lies in exactly one item of every
  neuron tile of (expert, p) - or in one item per half of the tile where the plan cut it in two -, and every
  row of H that an item of the second GEMM reads is written (computed or zero-filled) by exactly one item;
* second GEMM (Eq. 3): every row lies in exactly one (row range, column tile) group, the group's K ranges
  tile the partition's K stages without gap or overlap, exactly one of them writes the per-pair output and
  the others write distinct partial-output tiles, and the group sums over every partition a row of it keeps.
"""
import numpy as np
import pytest

from synth import make_layer
from gpu_util import make_gpu_layer, to_dev
from plan_cover import check_cover
from test_gpu_forward import spec_of, resolve_tau

pytestmark = pytest.mark.gpu

CASES = [
    # name, spec, tau, tall_items
    ("plain_tiles", spec_of(T=700, D=256, F=512, E=4, K=2, P=2, seed=80), 0.0, 0),
    ("drop_monotone", spec_of(T=900, D=128, F=1024, E=4, K=2, P=4, seed=81), "rate0.25", 0),
    ("drop_general_masks", spec_of(T=800, D=128, F=1024, E=4, K=3, P=4, seed=82), "ragged", 1),
    ("tall_forced", spec_of(T=540, D=128, F=512, E=4, K=2, P=2, seed=60), 0.0, 1),
    ("tall_priced", spec_of(T=1080, D=128, F=4096, E=8, K=2, P=4, seed=67), 0.0, 0),
    ("tall_under_drop", spec_of(T=560, D=128, F=1024, E=4, K=2, P=4, seed=63), "rate0.25", 1),
    ("shared_experts", spec_of(T=270, D=128, F=256, E=4, K=2, P=2, n_shared=1, F_sh=256, seed=65), 0.0, 1),
    ("decode_split_and_halves", spec_of(T=24, D=512, F=2048, E=8, K=2, P=2, seed=83), 0.0, 0),
    ("last_round_split", spec_of(T=8500, D=1024, F=2048, E=4, K=2, P=2, seed=45), 0.0, 0),
    ("half_full_last_neuron_tile", spec_of(T=540, D=128, F=384, E=4, K=2, P=2, seed=66), "rate0.25", 0),
    ("resident_window", spec_of(T=1500, D=128, F=512, E=8, K=2, P=2, seed=84, resident=(2, 7)), "rate0.25", 0),
]


@pytest.mark.parametrize("name,spec,tau_kind,tall_items", CASES, ids=[c[0] for c in CASES])
def test_work_lists_cover_every_kept_unit_once(oracle, name, spec, tau_kind, tall_items):
    import torch
    t = make_layer(spec)
    tau = resolve_tau(oracle, spec, t, tau_kind)
    layer, dev = make_gpu_layer(spec, t, tall_items=tall_items)
    assert layer.uses_mfma
    layer.forward(dev["x"], dev["logits"], to_dev(tau))
    torch.cuda.synchronize()
    plan = {k: (v.cpu().numpy() if hasattr(v, "cpu") else v) for k, v in layer.plan(spec.T).items()}
    layer.close()

    check_cover(plan, name=name, T=spec.T, D=spec.D, F=spec.F, P=spec.P, E_res=spec.hi - spec.lo, n_shared=spec.n_shared, F_sh=spec.F_sh)
