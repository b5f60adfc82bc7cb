#!/usr/bin/env python3
"""Benchmark of the DualSparse-MoE layer forward on one MI355X.

One "step" = one moe_dualsparse_forward call (route+mask, row lists, GEMM-1, GEMM-2, combine) on
the Mixtral-8x7B-shaped synthetic layer (T=4096, D=4096, E=8, F=14336, top-2, P=4) with the inputs
and packed weights already resident in HBM.  The headline value is tokens/s at about 25 % unit
drop; the same line carries the 0 / 25 / 50 % sweep (tokens/s, algorithmic TFLOP/s, fraction of the
bf16 MFMA peak), the roofline of the dominant kernel and the fp64 CPU oracle timed on a token
sample of the same workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C2] [--sample S] [--no-cpu] [--core-only] [--tokens T]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA, vendor figure
HBM_PEAK_GBS = 8000.0      # MI355X HBM3E, vendor figure


def log(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


def read_traffic(workload):
    """HBM bytes per GEMM-1 launch from the committed rocprofv3 counter summary, if there is one."""
    path = os.path.join(ROOT, "profiles", "gemm1_mfma_kernel_%s_hbm_traffic.txt" % workload)
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":", 1)[1])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="C2", choices=["C2", "C3", "C4", "C5"])
    ap.add_argument("--sample", type=int, default=0, help="tokens for the CPU oracle leg (0 = per workload)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--tokens", type=int, default=0, help="batch size instead of the workload's own (e.g. 64: a decode step)")
    ap.add_argument("--core-only", action="store_true",
                    help="only the layer's forward pass (no reconstruction / threshold selection / decode / router / "
                         "transformation timings): what the rocprofv3 summaries are taken from")
    ap.add_argument("--rates", default="0,0.25,0.5")
    ap.add_argument("--primary-rate", type=float, default=0.25)
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from synth import LAYERS, make_layer
    import paper_2508_18376_amd as ds
    from paper_2508_18376_amd.thresholds import tau_for_drop_rate, tau_capping_rows

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    spec = LAYERS[args.workload]
    if args.tokens:
        spec = spec.with_(T=args.tokens)  # same layer, another batch size (decode-sized batches: 16..256)
    K, W = args.steps, args.warmup

    t0 = time.time()
    host = make_layer(spec, threads=16)
    log("generated %s on the host in %.1f s" % (spec.name, time.time() - t0))

    def up(a):
        if a is None:
            return None
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)
        return torch.from_numpy(a).to(dev)

    layer = ds.DualSparseLayer(d_model=spec.D, d_ff=spec.F, n_experts=spec.E, top_k=spec.K, n_part=spec.P,
                               max_tokens=spec.T, dtype=spec.dtype, n_shared=spec.n_shared, d_ff_shared=spec.F_sh,
                               expert_lo=spec.lo, expert_hi=spec.hi)
    assert layer.uses_mfma, "the benchmark layer must run on the MFMA path"
    x, logits = up(host["x"]), up(host["logits"])
    wdev = {k: up(host.get(k)) for k in ("w1", "w3", "w2", "sh_w1", "sh_w3", "sh_w2", "perm")}
    t0 = time.time()
    layer.partition_weights(wdev["w1"], wdev["w3"], wdev["w2"], perm=wdev["perm"], sh_w1=wdev["sh_w1"], sh_w3=wdev["sh_w3"],
                            sh_w2=wdev["sh_w2"])
    torch.cuda.synchronize()
    log("moe_partition_weights: %.3f s" % (time.time() - t0))
    del wdev
    torch.cuda.empty_cache()

    # normalised scores from the GPU's own routing (renorm context, tau = 0) -> thresholds per rate
    rctx = ds.dsmoe_create(d_model=spec.D, d_ff=spec.F, n_experts=spec.E, top_k=spec.K, n_part=spec.P, max_tokens=spec.T,
                           dtype=1, expert_lo=spec.lo, expert_hi=spec.hi, renorm_combine=1)
    n_pairs = spec.T * spec.K
    r_idx = torch.empty(n_pairs, dtype=torch.int32, device=dev)
    r_w = torch.empty(n_pairs, dtype=torch.float32, device=dev)
    r_keep = torch.empty(n_pairs, dtype=torch.uint8, device=dev)
    r_gc = torch.empty(spec.E * spec.P, dtype=torch.int32, device=dev)
    tau0 = torch.zeros((spec.E, spec.P), dtype=torch.float32, device=dev)
    ds.moe_route_and_mask(rctx, logits, spec.T, tau0, r_idx, r_w, r_keep, r_gc)
    torch.cuda.synchronize()
    n_all = r_w.cpu().numpy().reshape(spec.T, spec.K)
    idx_all = r_idx.cpu().numpy().reshape(spec.T, spec.K)
    resident = (idx_all >= spec.lo) & (idx_all < spec.hi)
    n_res = n_all[resident]

    def tau_for(rate):
        tab = np.tile(tau_for_drop_rate(n_res, spec.P, rate)[None, :], (spec.E, 1)).astype(np.float32)
        if spec.name == "C5":  # load-aware cap: the hot expert keeps at most 1.25 x the balanced share of rows
            cap = int(1.25 * spec.T * spec.K / spec.E)
            for e in range(spec.lo, spec.hi):
                ne = n_all[idx_all == e]
                if ne.size > cap:
                    tab[e] = np.maximum(tab[e], tau_capping_rows(ne, spec.P, cap))
        return tab

    def kept_units(tau_dev):
        ds.moe_route_and_mask(rctx, logits, spec.T, tau_dev, r_idx, r_w, r_keep, r_gc)
        torch.cuda.synchronize()
        return int(r_gc.sum().item())

    Fp = spec.F // spec.P
    unit_flops = 6.0 * spec.D * Fp
    shared_flops = 6.0 * spec.D * spec.F_sh * spec.n_shared * spec.T
    total_units = int(resident.sum()) * spec.P
    y = torch.empty((spec.T, spec.D), dtype=torch.bfloat16, device=dev)
    stream = torch.cuda.current_stream()

    def run_steps(tau_dev, n):
        for _ in range(n):
            ds.moe_dualsparse_forward(layer.ctx, layer.packed, x, logits, tau_dev, spec.T, y, layer.workspace, stream)

    def timed(tau_dev, profile_level):
        run_steps(tau_dev, W)
        torch.cuda.synchronize()
        if profile_level:
            ds.dsmoe_profile_begin(layer.ctx, profile_level, K)
        torch.cuda.synchronize()
        t_start = time.perf_counter()
        run_steps(tau_dev, K)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t_start
        kms = None
        if profile_level:
            kms, calls = ds.dsmoe_profile_end(layer.ctx)
            assert calls == K
        return dt / K * 1e3, kms

    rates = [float(r) for r in args.rates.split(",")]
    if args.primary_rate not in rates:
        rates.append(args.primary_rate)
    sweep = []
    primary = None
    for rate in rates:
        tab = tau_for(rate)
        tau_dev = torch.from_numpy(tab).to(dev)
        units = kept_units(tau_dev)
        is_primary = abs(rate - args.primary_rate) < 1e-9
        ms, kms = timed(tau_dev, 1 if is_primary else 0)
        flops = unit_flops * units + shared_flops
        # with shared experts the paper counts them in the denominator (Sec. 5.1): dropped / (routed + shared)
        shared_units = spec.T * spec.n_shared * spec.P * (spec.F_sh / spec.F) if spec.n_shared else 0.0
        rec = {"target_drop": rate, "drop_rate": 1.0 - units / max(total_units, 1), "kept_units": units,
               "drop_rate_incl_shared": (total_units - units) / max(total_units + shared_units, 1),
               "ms_per_step": ms, "tokens_per_s": spec.T / (ms * 1e-3), "tflops": flops / (ms * 1e-3) / 1e12,
               "frac_bf16_peak": flops / (ms * 1e-3) / 1e12 / BF16_PEAK_TFLOPS, "tau": [float(v) for v in tab[spec.lo]]}
        sweep.append(rec)
        log("rate %.3f: %.3f ms/step, %.0f tokens/s, %.1f TFLOP/s (%.1f %% of bf16 peak), realised drop %.3f"
            % (rate, ms, rec["tokens_per_s"], rec["tflops"], 100 * rec["frac_bf16_peak"], rec["drop_rate"]))
        if is_primary:
            primary = dict(rec)
            primary["gemm1_ms"] = kms["gemm1"]
            primary["tau_table"] = tab
            primary["tau_dev"] = tau_dev
    # per-kernel table (separate pass with events between all kernels)
    _, kms_all = timed(primary["tau_dev"], 2)
    units = primary["kept_units"]
    pairs_kept = None
    plan = layer.plan(spec.T)
    pairs_kept = int((plan["pair_row"] >= 0).sum().item())
    bytes_route = spec.T * spec.E * 4 + spec.T * spec.K * 9
    bytes_scatter = spec.T * spec.K * 9 + pairs_kept * 5
    bytes_combine = pairs_kept * spec.D * 4 + spec.T * spec.D * 2 + spec.T * spec.K * 8 \
        + (spec.T * spec.D * 4 if spec.n_shared else 0)
    g1_flops = 4.0 * spec.D * Fp * units + 4.0 * spec.D * spec.F_sh * spec.n_shared * spec.T
    g2_flops = 2.0 * spec.D * Fp * units + 2.0 * spec.D * spec.F_sh * spec.n_shared * spec.T
    kernels = {k: {"ms": v} for k, v in kms_all.items()}
    kernels["route_mask"]["GBps"] = bytes_route / (kms_all["route_mask"] * 1e-3) / 1e9
    kernels["scatter"]["GBps"] = bytes_scatter / (kms_all["scatter"] * 1e-3) / 1e9
    kernels["combine"]["GBps"] = bytes_combine / (kms_all["combine"] * 1e-3) / 1e9
    kernels["gemm1"]["tflops"] = g1_flops / (kms_all["gemm1"] * 1e-3) / 1e12
    kernels["gemm2"]["tflops"] = g2_flops / (kms_all["gemm2"] * 1e-3) / 1e12

    g1_ach = g1_flops / (primary["gemm1_ms"] * 1e-3) / 1e12
    roofline = {"kernel": "gemm1_mfma_kernel", "bound": "mfma", "achieved": g1_ach, "peak": BF16_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": g1_ach / BF16_PEAK_TFLOPS, "traffic": read_traffic(spec.name),
                "avg_launch_ms": primary["gemm1_ms"], "flops_per_launch": g1_flops}

    reconstruction = selection = router = transform = None
    decode = []
    if not args.core_only:
        # reconstruction step that precedes the path (Sec. 4.2 b): importance of this batch used as the
        # calibration set (every routed pair, no drops) and the order made from it; timed on its own
        def ev_ms(fn, n):
            fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(n):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / n

        imp = torch.empty((spec.E_res, spec.F), dtype=torch.float32, device=dev)
        perm_out = torch.empty((spec.E_res, spec.F), dtype=torch.int32, device=dev)
        n_rec = max(2, K // 5)
        rec_ms = ev_ms(lambda: ds.moe_profile_importance(layer.ctx, layer.packed, x, logits, spec.T, 3, imp, layer.workspace,
                                                         stream), n_rec)
        perm_ms = ev_ms(lambda: ds.moe_importance_to_perm(layer.ctx, imp, perm_out, stream), n_rec)
        rec_flops = 4.0 * spec.D * spec.F * int(resident.sum())
        reconstruction = {"profile_importance_ms": rec_ms, "profile_importance_tflops": rec_flops / (rec_ms * 1e-3) / 1e12,
                          "importance_to_perm_ms": perm_ms, "calibration_tokens": spec.T, "metric": 3}
        log("reconstruction: importance of %d tokens %.3f ms (%.0f TFLOP/s), order %.3f ms"
            % (spec.T, rec_ms, reconstruction["profile_importance_tflops"], perm_ms))

        # load-aware threshold selection on the device (Sec. 4.3): the step that can feed `tau` every batch
        tau_sel = torch.empty((spec.E, spec.P), dtype=torch.float32, device=dev)
        pairs_sel = torch.empty((spec.E,), dtype=torch.int32, device=dev)
        tau_max_dev = torch.from_numpy(np.ascontiguousarray(primary["tau_table"][spec.lo])).to(dev)
        cap_rows = int(1.25 * spec.T * spec.K / spec.E)
        sel_ms = ev_ms(lambda: ds.moe_select_thresholds(layer.ctx, logits, spec.T, tau_max_dev, 1, cap_rows, tau_sel, pairs_sel,
                                                        layer.workspace, stream), max(10, K))
        off_bins = [0] if spec.P == 1 else [round(41 * (2 * p - (spec.P - 1)) / (spec.P - 1)) for p in range(spec.P)]
        stats_sel = torch.empty((2,), dtype=torch.int32, device=dev)
        rate_ms = ev_ms(lambda: ds.moe_thresholds_for_drop_rate(layer.ctx, logits, spec.T, args.primary_rate, off_bins, tau_sel,
                                                                stats_sel, layer.workspace, stream), max(10, K))
        st = stats_sel.cpu().numpy()
        selection = {"select_thresholds_ms": sel_ms, "group_size": 1, "row_cap": cap_rows,
                     "thresholds_for_drop_rate_ms": rate_ms, "target_drop": args.primary_rate,
                     "device_chosen_drop": float(st[0]) / max(float(st[1]), 1.0)}
        log("threshold selection (ratio rule + row cap %d): %.4f ms; thresholds for %.0f %% drop: %.4f ms (realised %.1f %%)"
            % (cap_rows, sel_ms, 100 * args.primary_rate, rate_ms, 100 * selection["device_chosen_drop"]))

        # gating product x W_g in front of the path (Sec. 3.1, first equation) and the complete transformation
        from synth import make_router
        wg_host = make_router(spec)
        router_packed = torch.empty(max(ds.dsmoe_router_packed_bytes(layer.ctx), 16), dtype=torch.uint8, device=dev)
        ds.moe_pack_router(layer.ctx, up(wg_host), router_packed, stream)
        lg_out = torch.empty((spec.T, spec.E), dtype=torch.float32, device=dev)
        router_ms = ev_ms(lambda: ds.moe_router_logits(layer.ctx, router_packed, x, spec.T, lg_out, stream), max(10, K))
        routed_ms = ev_ms(lambda: ds.moe_dualsparse_forward_routed(layer.ctx, layer.packed, router_packed, x, primary["tau_dev"],
                                                                   spec.T, y, None, layer.workspace, stream), max(5, K // 2))
        router_bytes = spec.T * spec.D * 2 + spec.T * spec.E * 4
        router = {"router_logits_ms": router_ms, "GBps": router_bytes / (router_ms * 1e-3) / 1e9,
                  "forward_routed_ms": routed_ms}
        log("router x W_g: %.4f ms (%.0f GB/s of x); layer driven by those logits (another routing, same tau table) %.3f ms"
            % (router_ms, router["GBps"], routed_ms))
        del lg_out
        w_dev = {k: up(host[k]) for k in ("w1", "w3", "w2")}
        w_out = {k: torch.empty_like(v) for k, v in w_dev.items()}
        wg_dev, wg_out = up(wg_host), torch.empty((spec.D, spec.E * spec.P), dtype=torch.bfloat16, device=dev)
        perm_dev = up(host["perm"])
        tr_ms = ev_ms(lambda: ds.moe_transform_complete(layer.ctx, wg_dev, w_dev["w1"], w_dev["w3"], w_dev["w2"], perm_dev, wg_out,
                                                        w_out["w1"], w_out["w3"], w_out["w2"], layer.workspace, stream), 2)
        w_bytes = sum(v.numel() * 2 for v in w_dev.values())
        transform = {"transform_complete_ms": tr_ms, "GBps": 2 * w_bytes / (tr_ms * 1e-3) / 1e9}
        log("complete transformation of %.2f GB of weights: %.2f ms (%.0f GB/s read + write)" % (w_bytes / 1e9, tr_ms, transform["GBps"]))
        del w_dev, w_out

        # decode-sized batches of the same layer (weight streaming regime): the first T tokens of the batch
        decode = []
        w_unit_bytes = 3 * spec.D * Fp * 2
        for Td in (16, 64, 256):
            if Td > spec.T:
                continue
            xd, ld = x[:Td].contiguous(), logits[:Td].contiguous()
            res_d = resident[:Td]
            tab = np.tile(tau_for_drop_rate(n_all[:Td][res_d], spec.P, args.primary_rate)[None, :], (spec.E, 1)).astype(np.float32)
            tau_d = torch.from_numpy(tab).to(dev)
            ds.moe_route_and_mask(rctx, ld, Td, tau_d, r_idx, r_w, r_keep, r_gc)
            torch.cuda.synchronize()
            gc = r_gc.cpu().numpy()
            active = int((gc > 0).sum())
            wbytes = active * w_unit_bytes + 3 * spec.D * spec.F_sh * spec.n_shared * 2
            yd = torch.empty((Td, spec.D), dtype=torch.bfloat16, device=dev)
            fn = lambda: ds.moe_dualsparse_forward(layer.ctx, layer.packed, xd, ld, tau_d, Td, yd, layer.workspace, stream)
            for _ in range(W):
                fn()
            torch.cuda.synchronize()
            t_start = time.perf_counter()
            for _ in range(K):
                fn()
            torch.cuda.synchronize()
            ms_d = (time.perf_counter() - t_start) / K * 1e3
            decode.append({"tokens": Td, "ms_per_step": ms_d, "tokens_per_s": Td / (ms_d * 1e-3), "active_sub_experts": active,
                           "kept_units": int(gc.sum()), "weight_bytes": wbytes, "GBps": wbytes / (ms_d * 1e-3) / 1e9,
                           "frac_hbm_peak": wbytes / (ms_d * 1e-3) / 1e9 / 8000.0})
            log("decode T=%d: %.3f ms/step, weights of %d active sub-experts %.2f GB -> %.0f GB/s (%.0f %% of 8 TB/s)"
                % (Td, ms_d, active, wbytes / 1e9, decode[-1]["GBps"], 100 * decode[-1]["frac_hbm_peak"]))

    # proportionality of the time saved at the primary rate, against the 0 % run
    t_zero = next((r["ms_per_step"] for r in sweep if r["target_drop"] == 0.0), None)
    prop = None
    if t_zero:
        prop = {"time_reduction": (t_zero - primary["ms_per_step"]) / t_zero, "drop_rate": primary["drop_rate"]}
        prop["frac_of_proportional"] = prop["time_reduction"] / max(primary["drop_rate"], 1e-9)

    # CPU oracle leg: the same layer and thresholds on a seeded token sample, all host cores
    cpu = None
    check = None
    if not args.no_cpu:
        import oracle
        S = args.sample or {"C2": 1536, "C3": 8192, "C4": 6144, "C5": 2048}[spec.name]  # about 10 s of oracle time each
        S = min(S, spec.T)
        tok = np.sort(np.random.default_rng(12345).choice(spec.T, size=S, replace=False)).astype(np.int32)
        t0 = time.time()
        y_ref = oracle.forward(host["x"], host["logits"], host["w1"], host["w3"], host["w2"], primary["tau_table"], spec.K,
                               spec.P, perm=host["perm"], sh_w1=host.get("sh_w1"), sh_w3=host.get("sh_w3"),
                               sh_w2=host.get("sh_w2"), lo=spec.lo, hi=spec.hi, tokens=tok)
        dt = time.time() - t0
        cpu_model = ""
        try:
            for line in open("/proc/cpuinfo"):
                if line.startswith("model name"):
                    cpu_model = line.split(":", 1)[1].strip()
                    break
        except OSError:
            pass
        cpu = {"value": S / dt, "unit": "tokens/s", "cores": oracle.n_threads(), "kind": "oracle",
               "host": {"nproc": os.cpu_count(), "cpu": cpu_model},
               "note": "the oracle as it stands, untuned: a reported baseline, not a competitor",
               "sample": "%d of %d tokens (seeded), whole layer per token, %.1f s" % (S, spec.T, dt)}
        run_steps(primary["tau_dev"], 1)
        torch.cuda.synchronize()
        y_s = y[torch.from_numpy(tok.astype(np.int64)).to(dev)].to(torch.float32).cpu().numpy().astype(np.float64)
        rms = float(np.sqrt(np.mean(y_ref ** 2)))
        aerr = np.abs(y_s - y_ref)
        # the bf16 output format costs up to 2^-8 |y| by itself; the rest is the computation's error
        beyond = aerr - 2.0 ** -8 * np.abs(y_ref)
        check = {"elements": int(aerr.size), "rms_err_over_rms": float(np.sqrt(np.mean(aerr ** 2)) / rms),
                 "elements_beyond_tolerance": int((beyond > 2e-2 * rms).sum()),
                 "sample_max_err_over_rms": float(aerr.max() / rms),
                 "sample_max_err_beyond_bf16_output_rounding_over_rms": float((aerr - 2.0 ** -8 * np.abs(y_ref)).max() / rms),
                 "tolerance": 2e-2}
        log("oracle: %.2f tokens/s on %d threads; GPU vs oracle on the sample: max |err| %.4f x RMS, %.4f x RMS beyond the "
            "rounding of the bf16 output (bar 0.02), %d elements over the bar" % (
                cpu["value"], cpu["cores"], check["sample_max_err_over_rms"],
                check["sample_max_err_beyond_bf16_output_rounding_over_rms"], check["elements_beyond_tolerance"]))

    out = {
        "metric": "MoE-layer tokens/s + MFMA TFLOP/s vs bf16 peak at 0/25/50% drop",
        "value": primary["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": primary["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s: T=%d D=%d E=%d F=%d top-%d P=%d%s, tau for ~%d%% unit drop (realised %.1f%%)" % (
            spec.name, spec.T, spec.D, spec.E, spec.F, spec.K, spec.P,
            (" + %d shared x %d" % (spec.n_shared, spec.F_sh)) if spec.n_shared else "",
            round(100 * args.primary_rate), 100 * primary["drop_rate"]),
            "resident_experts": [spec.lo, spec.hi], "tokens": spec.T},
        "tflops": primary["tflops"], "frac_bf16_peak": primary["frac_bf16_peak"],
        "sweep": sweep, "proportionality": prop, "kernels": kernels,
        "kernels_note": "HIP-event intervals around each launch of a separate timing pass: every entry carries about 4 us of "
                        "event-to-event gap (an empty interval reads 4-5 us); kernel durations proper are in profiles/",
        "reconstruction": reconstruction, "threshold_selection": selection, "decode": decode, "router": router, "complete_transformation": transform,
        "roofline": roofline, "cpu_baseline": cpu, "check": check,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
