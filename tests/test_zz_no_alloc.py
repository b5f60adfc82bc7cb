"""moe_dualsparse_forward_static (the entry point for callers that cannot allocate device memory)
against moe_dualsparse_forward, through the C ABI: two calls in a row on one GPU, the second with
a smaller batch, so that the second call runs over what the first one left in the library's
static scratch array.  The two entry points share their kernels, so the outputs must be equal bit
for bit; both are also held to the oracle's bar.  Covers the MFMA path (bf16, shared experts) and
the generic path (fp32), the refusal of a batch that does not fit, and T = 0.
"""

import numpy as np
import pytest

from synth import LayerSpec, make_layer
from gpu_util import GUARD, make_gpu_layer, to_dev, to_host64, pick_tau, tau_table, assert_output_close

pytestmark = pytest.mark.gpu

CASES = [
    LayerSpec("static_bf16", T=700, D=256, F=512, E=8, K=2, P=2, dtype="bf16", seed=21, n_shared=1, F_sh=256),
    LayerSpec("static_f32", T=300, D=96, F=120, E=6, K=3, P=3, dtype="f32", seed=22, x_std=0.5, w_std=0.1),
]


@pytest.mark.parametrize("spec", CASES, ids=[c.name for c in CASES])
def test_static_scratch_forward_matches_workspace_forward(oracle, spec):
    import torch
    import paper_2508_18376_amd as ds
    t = make_layer(spec)
    r0 = oracle.route(t["logits"], spec.K, spec.P, np.zeros((spec.E, spec.P), np.float32))
    tau = tau_table(spec, pick_tau(r0.n, spec.P, 0.3))
    assert oracle.route(t["logits"], spec.K, spec.P, tau).min_margin > GUARD
    layer, dev = make_gpu_layer(spec, t)
    assert layer.uses_mfma == (spec.dtype == "bf16")
    tau_dev = to_dev(tau)
    stream = torch.cuda.current_stream()
    assert 0 < ds.dsmoe_static_workspace_need(layer.ctx, spec.T) <= ds.DSMOE_STATIC_SCRATCH_BYTES

    # set-up call (T = 0): looks the array up, launches nothing
    ds.moe_dualsparse_forward_static(layer.ctx, layer.packed, None, None, tau_dev, 0, None, stream)

    for T in (spec.T, 130):  # the second, smaller call finds the first one's leftovers in the array
        print("static forward: %s T=%d" % (spec.name, T), flush=True)
        x, lg = dev["x"][:T].contiguous(), dev["logits"][:T].contiguous()
        y_ws = layer.forward(x, lg, tau_dev)
        y_st = torch.full_like(y_ws, float("nan"))
        ds.moe_dualsparse_forward_static(layer.ctx, layer.packed, x, lg, tau_dev, T, y_st, stream)
        torch.cuda.synchronize()
        assert torch.equal(y_st.view(torch.int16 if spec.dtype == "bf16" else torch.int32),
                           y_ws.view(torch.int16 if spec.dtype == "bf16" else torch.int32))
        y_ref = oracle.forward(t["x"][:T], t["logits"][:T], t["w1"], t["w3"], t["w2"], tau, spec.K, spec.P, perm=t["perm"],
                               sh_w1=t.get("sh_w1"), sh_w3=t.get("sh_w3"), sh_w2=t.get("sh_w2"))
        assert_output_close(to_host64(y_st, spec.dtype), y_ref, spec.dtype)
    layer.close()


def test_static_scratch_forward_refuses_what_does_not_fit():
    """A batch whose workspace exceeds the array is refused before anything is launched."""
    import torch
    import paper_2508_18376_amd as ds
    T = 200000
    ctx = ds.dsmoe_create(d_model=256, d_ff=512, n_experts=8, top_k=2, n_part=2, max_tokens=T, dtype=1)
    assert ds.dsmoe_static_workspace_need(ctx, T) > ds.DSMOE_STATIC_SCRATCH_BYTES
    dummy = torch.zeros(64, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(ds.DsmoeError) as ei:
        ds.moe_dualsparse_forward_static(ctx, dummy, dummy, dummy, dummy, T, dummy, torch.cuda.current_stream())
    assert ei.value.status == -3
    ds.dsmoe_destroy(ctx)
