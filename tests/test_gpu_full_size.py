"""GPU parity at the benchmark's full sizes (the four bf16 layers), in the launch configuration
bench.py times: routing and masks bit-exact for every token, layer output against the fp64 oracle
on a stratified token sample (every resident expert and every keep pattern that occurs is hit),
and whole-tensor properties for the rows the oracle does not compute (finite, same scale, exact
zeros where every unit of a token is dropped).
"""
import numpy as np
import pytest

from synth import LAYERS, make_layer
from gpu_util import GUARD, make_gpu_layer, to_dev, to_host64, pick_tau, tau_table, assert_output_close

pytestmark = pytest.mark.gpu

# (layer, target drop rate of routed units, tokens in the oracle sample)
CASES = [("C2", 0.25, 96), ("C2", 0.0, 48), ("C3", 0.25, 384), ("C3", 0.5, 256), ("C4", 1.0 / 3.0, 320), ("C5", 0.25, 96)]


def stratified_sample(spec, route, n, seed=7):
    rng = np.random.default_rng(seed)
    bits = route.keep_bits
    chosen = []
    per_cell = max(1, n // max(1, (spec.hi - spec.lo) * spec.P * 2))
    for e in range(spec.lo, spec.hi):
        for pat in np.unique(bits[route.idx == e]):
            toks = np.unique(np.nonzero((route.idx == e) & (bits == pat))[0])
            if toks.size:
                chosen.extend(rng.choice(toks, size=min(per_cell, toks.size), replace=False).tolist())
    dead = np.nonzero(bits.sum(axis=1) == 0)[0]
    if dead.size:
        chosen.extend(dead[:4].tolist())
    chosen = list(dict.fromkeys(chosen))
    if len(chosen) < n:
        rest = np.setdiff1d(np.arange(spec.T), np.array(chosen, dtype=np.int64))
        chosen.extend(rng.choice(rest, size=n - len(chosen), replace=False).tolist())
    return np.sort(np.array(chosen[:max(n, 1)], dtype=np.int32))


@pytest.mark.parametrize("name,rate,n_sample", CASES, ids=["%s-%d%%" % (c[0], round(100 * c[1])) for c in CASES])
def test_full_size_layer(oracle, name, rate, n_sample):
    import torch
    spec = LAYERS[name]
    t = make_layer(spec, threads=16)
    r0 = oracle.route(t["logits"], spec.K, spec.P, np.zeros((spec.E, spec.P), np.float32), spec.lo, spec.hi)
    res = (r0.idx >= spec.lo) & (r0.idx < spec.hi)
    tau = tau_table(spec, pick_tau(r0.n[res], spec.P, rate))
    if name == "C5":  # load-aware cap on the hot expert: at most 1.25 x the balanced share of rows
        cap = int(1.25 * spec.T * spec.K / spec.E)
        for e in range(spec.lo, spec.hi):
            ne = r0.n[r0.idx == e]
            if ne.size > cap:
                tau[e] = np.maximum(tau[e], pick_tau(ne, spec.P, 1.0 - cap / ne.size, window=0.002))
    ref = oracle.route(t["logits"], spec.K, spec.P, tau, spec.lo, spec.hi)
    assert ref.min_margin > GUARD, ref.min_margin
    if rate > 0:
        units = res.sum() * spec.P
        assert abs(1.0 - ref.keep.sum() / units - rate) < 0.02 or name == "C5"

    layer, dev = make_gpu_layer(spec, t)
    assert layer.uses_mfma
    tau_dev = to_dev(tau)
    idx, w, keep, gc = layer.route_and_mask(dev["logits"], tau_dev)
    y = layer.forward(dev["x"], dev["logits"], tau_dev)
    torch.cuda.synchronize()
    # routing and masks: every token, bit-exact
    np.testing.assert_array_equal(idx.cpu().numpy(), ref.idx)
    np.testing.assert_array_equal(keep.cpu().numpy(), ref.keep_bits)
    np.testing.assert_array_equal(gc.cpu().numpy().astype(np.int64), ref.group_count)
    np.testing.assert_allclose(w.cpu().numpy().astype(np.float64), ref.g, rtol=2e-6)
    plan = layer.plan(spec.T)
    np.testing.assert_array_equal(plan["keep_bits"].cpu().numpy(), ref.keep_bits)
    nrows = plan["expert_nrows"].cpu().numpy()
    for i, e in enumerate(range(spec.lo, spec.hi)):
        assert nrows[i] == int(((ref.idx == e) & (ref.keep_bits != 0)).sum())

    # layer output on the sample
    tok = stratified_sample(spec, ref, n_sample)
    y_ref = oracle.forward(t["x"], t["logits"], t["w1"], t["w3"], t["w2"], tau, spec.K, spec.P, perm=t["perm"],
                           sh_w1=t.get("sh_w1"), sh_w3=t.get("sh_w3"), sh_w2=t.get("sh_w2"), lo=spec.lo, hi=spec.hi, tokens=tok)
    y_all = to_host64(y, "bf16")
    assert_output_close(y_all[tok], y_ref, "bf16")

    # the other rows: finite, same scale, exact zeros for fully dropped tokens
    assert np.isfinite(y_all).all()
    rms_all = np.sqrt(np.mean(y_all ** 2))
    rms_ref = np.sqrt(np.mean(y_ref ** 2))
    assert abs(rms_all / rms_ref - 1.0) < 0.15, (rms_all, rms_ref)
    if spec.n_shared == 0:
        dead = ref.keep_bits.sum(axis=1) == 0
        assert np.all(y_all[dead] == 0.0)
        assert np.all(np.abs(y_all[~dead]).max(axis=1) > 0)
    layer.close()


# decode-sized batches of the full-size layers: the weight-streaming regime (split K in GEMM-2,
# halved GEMM-1 items, half-empty neuron tiles as first halves), every token against the oracle
DECODE_CASES = [("C2", 64), ("C2", 16), ("C3", 48), ("C4", 64), ("C5", 32)]


@pytest.mark.parametrize("name,T", DECODE_CASES, ids=["%s-%d" % c for c in DECODE_CASES])
def test_full_size_layer_decode_batch(oracle, name, T):
    import torch
    spec = LAYERS[name].with_(T=T)
    t = make_layer(spec, threads=16)
    r0 = oracle.route(t["logits"], spec.K, spec.P, np.zeros((spec.E, spec.P), np.float32), spec.lo, spec.hi)
    res = (r0.idx >= spec.lo) & (r0.idx < spec.hi)
    ref = tau = None
    for rate in (0.25, 0.27, 0.23, 0.29, 0.21, 0.31):  # few scores: take the first rate whose thresholds clear the guard band
        tau = tau_table(spec, pick_tau(r0.n[res], spec.P, rate, window=0.02))
        ref = oracle.route(t["logits"], spec.K, spec.P, tau, spec.lo, spec.hi)
        if ref.min_margin > GUARD:
            break
    assert ref.min_margin > GUARD, ref.min_margin
    layer, dev = make_gpu_layer(spec, t)
    assert layer.uses_mfma
    tau_dev = to_dev(tau)
    idx, w, keep, gc = layer.route_and_mask(dev["logits"], tau_dev)
    y = layer.forward(dev["x"], dev["logits"], tau_dev)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(idx.cpu().numpy(), ref.idx)
    np.testing.assert_array_equal(keep.cpu().numpy(), ref.keep_bits)
    y_ref = oracle.forward(t["x"], t["logits"], t["w1"], t["w3"], t["w2"], tau, spec.K, spec.P, perm=t["perm"],
                           sh_w1=t.get("sh_w1"), sh_w3=t.get("sh_w3"), sh_w2=t.get("sh_w2"), lo=spec.lo, hi=spec.hi)
    assert_output_close(to_host64(y, "bf16"), y_ref, "bf16")
    layer.close()
