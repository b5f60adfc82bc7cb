#!/usr/bin/env python3
"""Benchmark of the DualSparse-MoE layer forward on one MI355X.

One "step" = one moe_dualsparse_forward call (route+mask, row lists, GEMM-1, GEMM-2, combine) with the
inputs and packed weights already resident in HBM.  The headline is the Mixtral-8x7B-shaped synthetic
layer (C2: T=4096, D=4096, E=8, F=14336, top-2, P=4): tokens/s at about 25 % unit drop, the 0 / 25 / 50 %
sweep (tokens/s, algorithmic TFLOP/s, fraction of the bf16 MFMA peak), the roofline of the dominant
kernel and the fp64 CPU oracle timed on a token sample of the same workload.  The same JSON line
carries, under "workloads", the fine-grained layer (C3: 0 / 12.5 / 25 / 50 %), the shared-plus-routed
layer (C4: about 25 % by the paper's definition) and the skewed expert-parallel share (C5: load-aware
thresholds with a row cap), each with its per-kernel split.

Every threshold table that is timed is chosen by the library itself on the device
(moe_thresholds_for_drop_rate, moe_select_thresholds) from the batch's own scores.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C2] [--no-cpu] [--core-only]
                    [--tokens T] [--rates 0,0.25,0.5] [--no-others]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 / fp16 MFMA, vendor figure
HBM_PEAK_GBS = 8000.0      # MI355X HBM3E, vendor figure


def log(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


def read_traffic(workload):
    """HBM-side bytes per GEMM-1 launch from the committed rocprofv3 counter summary of this workload
    (profiles/), or None: counters cannot be read from inside the timed run."""
    path = os.path.join(ROOT, "profiles", "gemm1_mfma_kernel_%s_hbm_traffic.txt" % workload)
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":", 1)[1])
    except OSError:
        pass
    return None


class Workload:
    """One synthetic layer on the GPU: packed weights, inputs, a routing-only context for counting."""

    def __init__(self, name, tokens, np, torch, ds, keep_host=False):
        from synth import LAYERS, make_layer
        self.np, self.torch, self.ds = np, torch, ds
        self.dev = torch.device("cuda:0")
        spec = LAYERS[name]
        if tokens:
            spec = spec.with_(T=tokens)  # same layer, another batch size (decode-sized batches: 16..256)
        self.spec = spec
        t0 = time.time()
        host = make_layer(spec, threads=16)
        log("generated %s on the host in %.1f s" % (spec.name, time.time() - t0))
        self.layer = ds.DualSparseLayer(d_model=spec.D, d_ff=spec.F, n_experts=spec.E, top_k=spec.K, n_part=spec.P,
                                        max_tokens=spec.T, dtype=spec.dtype, n_shared=spec.n_shared, d_ff_shared=spec.F_sh,
                                        expert_lo=spec.lo, expert_hi=spec.hi)
        assert self.layer.uses_mfma, "the benchmark layers run on the MFMA path"
        self.x, self.logits = self.up(host["x"]), self.up(host["logits"])
        wdev = {k: self.up(host.get(k)) for k in ("w1", "w3", "w2", "sh_w1", "sh_w3", "sh_w2", "perm")}
        t0 = time.time()
        self.layer.partition_weights(wdev["w1"], wdev["w3"], wdev["w2"], perm=wdev["perm"], sh_w1=wdev["sh_w1"],
                                     sh_w3=wdev["sh_w3"], sh_w2=wdev["sh_w2"])
        torch.cuda.synchronize()
        log("moe_partition_weights (%s): %.3f s" % (spec.name, time.time() - t0))
        del wdev
        torch.cuda.empty_cache()
        self.host = host if keep_host else None
        # a second context that only routes (normalised scores as weights), for unit counts
        self.rctx = ds.dsmoe_create(d_model=spec.D, d_ff=spec.F, n_experts=spec.E, top_k=spec.K, n_part=spec.P,
                                    max_tokens=spec.T, dtype=1, expert_lo=spec.lo, expert_hi=spec.hi, renorm_combine=1)
        n_pairs = spec.T * spec.K
        self.r_idx = torch.empty(n_pairs, dtype=torch.int32, device=self.dev)
        self.r_w = torch.empty(n_pairs, dtype=torch.float32, device=self.dev)
        self.r_keep = torch.empty(n_pairs, dtype=torch.uint8, device=self.dev)
        self.r_gc = torch.empty(spec.E * spec.P, dtype=torch.int32, device=self.dev)
        self.y = torch.empty((spec.T, spec.D), dtype=torch.bfloat16, device=self.dev)
        self.stream = torch.cuda.current_stream()
        tau0 = torch.zeros((spec.E, spec.P), dtype=torch.float32, device=self.dev)
        self.total_units = self.kept_units(tau0)  # resident routed units with nothing dropped
        self.Fp = spec.F // spec.P
        self.unit_flops = 6.0 * spec.D * self.Fp
        self.shared_flops = 6.0 * spec.D * spec.F_sh * spec.n_shared * spec.T
        # with shared experts the paper counts them in the denominator of the drop rate (Sec. 5.1)
        self.shared_units = spec.T * spec.n_shared * spec.P * (spec.F_sh / spec.F) if spec.n_shared else 0.0

    def up(self, a):
        np, torch = self.np, self.torch
        if a is None:
            return None
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).to(self.dev).view(torch.bfloat16)
        return torch.from_numpy(a).to(self.dev)

    def kept_units(self, tau_dev, T=None, logits=None):
        T = self.spec.T if T is None else T
        self.ds.moe_route_and_mask(self.rctx, self.logits if logits is None else logits, T, tau_dev, self.r_idx, self.r_w,
                                   self.r_keep, self.r_gc)
        self.torch.cuda.synchronize()
        return int(self.r_gc.sum().item())

    def tau_for_rate(self, rate, T=None, logits=None):
        """Threshold table for a target drop rate of the resident units, chosen on the device."""
        spec, torch = self.spec, self.torch
        if rate <= 0:
            return torch.zeros((spec.E, spec.P), dtype=torch.float32, device=self.dev)
        lg = self.logits if logits is None else logits
        tau, _ = self.layer.thresholds_for_drop_rate(lg if T is None else lg[:T].contiguous(), rate)
        return tau

    def tau_load_aware(self, tau_max_row, row_cap):
        """Sec. 4.3 on the device: thresholds scaled by the load ratio of each expert, and lifted where an
        expert would still keep more than row_cap pairs."""
        tau, pairs = self.layer.select_thresholds(self.logits, tau_max_row, group_size=1, row_cap=row_cap)
        return tau

    def run(self, tau_dev, n):
        for _ in range(n):
            self.ds.moe_dualsparse_forward(self.layer.ctx, self.layer.packed, self.x, self.logits, tau_dev, self.spec.T, self.y,
                                           self.layer.workspace, self.stream)

    def timed(self, tau_dev, K, W, profile_level=0):
        ds, torch = self.ds, self.torch
        self.run(tau_dev, W)
        torch.cuda.synchronize()
        if profile_level:
            ds.dsmoe_profile_begin(self.layer.ctx, profile_level, K)
        torch.cuda.synchronize()
        t_start = time.perf_counter()
        self.run(tau_dev, K)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t_start
        kms = None
        if profile_level:
            kms, calls = ds.dsmoe_profile_end(self.layer.ctx)
            assert calls == K
        return dt / K * 1e3, kms

    def sweep(self, cases, K, W, reps=3, profile_label=None):
        """Times every (label, tau) of `cases`: `reps` passes over the list, each pass W warm-up + K timed steps
        per case, so that the cases see the same clock and temperature drift; a case's figure is the median of
        its passes.  The case named profile_label also gets its GEMM-1 launches timed with HIP events (last pass)."""
        spec = self.spec
        units = [self.kept_units(tau) for _, tau in cases]
        samples = [[] for _ in cases]
        g1_ms = None
        for rep in range(reps):
            for i, (label, tau) in enumerate(cases):
                prof = 1 if (label == profile_label and rep == reps - 1) else 0
                ms, kms = self.timed(tau, K, W, prof)
                samples[i].append(ms)
                if prof:
                    g1_ms = kms["gemm1"]
        recs = []
        for i, (label, tau) in enumerate(cases):
            ms = sorted(samples[i])[len(samples[i]) // 2]
            flops = self.unit_flops * units[i] + self.shared_flops
            rec = {"case": label, "drop_rate": 1.0 - units[i] / max(self.total_units, 1), "kept_units": units[i],
                   "drop_rate_incl_shared": (self.total_units - units[i]) / max(self.total_units + self.shared_units, 1),
                   "ms_per_step": ms, "ms_per_step_passes": samples[i], "tokens_per_s": spec.T / (ms * 1e-3),
                   "tflops": flops / (ms * 1e-3) / 1e12, "frac_bf16_peak": flops / (ms * 1e-3) / 1e12 / BF16_PEAK_TFLOPS,
                   "flops": flops, "tau": [float(v) for v in tau[spec.lo].cpu().numpy()]}
            log("%s %s: %.3f ms/step (passes %s), %.0f tokens/s, %.1f TFLOP/s (%.1f %% of bf16 peak), realised drop %.3f"
                % (spec.name, label, ms, " ".join("%.3f" % v for v in samples[i]), rec["tokens_per_s"], rec["tflops"],
                   100 * rec["frac_bf16_peak"], rec["drop_rate"]))
            recs.append(rec)
        return recs, g1_ms

    def kernel_table(self, tau_dev, K, W):
        """Per-kernel split from HIP events between all launches (its own timing pass)."""
        spec = self.spec
        units = self.kept_units(tau_dev)
        _, kms = self.timed(tau_dev, K, W, 2)
        plan = self.layer.plan(spec.T)
        pairs_kept = int((plan["pair_row"] >= 0).sum().item())
        bytes_route = spec.T * spec.E * 4 + spec.T * spec.K * 9
        bytes_scatter = spec.T * spec.K * 9 + pairs_kept * 5
        bytes_combine = pairs_kept * spec.D * 4 + spec.T * spec.D * 2 + spec.T * spec.K * 8 \
            + (spec.T * spec.D * 4 if spec.n_shared else 0)
        g1_flops = 4.0 * spec.D * self.Fp * units + 4.0 * spec.D * spec.F_sh * spec.n_shared * spec.T
        g2_flops = 2.0 * spec.D * self.Fp * units + 2.0 * spec.D * spec.F_sh * spec.n_shared * spec.T
        kernels = {k: {"ms": v} for k, v in kms.items()}
        kernels["route_mask"]["GBps"] = bytes_route / (kms["route_mask"] * 1e-3) / 1e9
        kernels["scatter"]["GBps"] = bytes_scatter / (kms["scatter"] * 1e-3) / 1e9
        kernels["combine"]["GBps"] = bytes_combine / (kms["combine"] * 1e-3) / 1e9
        kernels["gemm1"]["tflops"] = g1_flops / (kms["gemm1"] * 1e-3) / 1e12
        kernels["gemm2"]["tflops"] = g2_flops / (kms["gemm2"] * 1e-3) / 1e12
        return kernels, g1_flops

    def close(self):
        self.ds.dsmoe_destroy(self.rctx)
        self.layer.close()
        del self.layer, self.x, self.logits, self.y
        self.torch.cuda.empty_cache()


def proportionality(zero, rec):
    """Time saved against the work removed, both relative to the run with nothing dropped."""
    saved = (zero["ms_per_step"] - rec["ms_per_step"]) / zero["ms_per_step"]
    removed = 1.0 - rec["flops"] / zero["flops"]
    return {"time_reduction": saved, "work_reduction": removed, "drop_rate": rec["drop_rate"],
            "frac_of_proportional": saved / max(removed, 1e-9)}


def other_workload(name, np, torch, ds, K, W):
    """The fine-grained (C3), shared-plus-routed (C4) and skewed expert-parallel (C5) layers."""
    w = Workload(name, 0, np, torch, ds)
    spec = w.spec
    todo = [("0%", w.tau_for_rate(0.0))]
    if name == "C3":
        for rate in (0.125, 0.25, 0.5):
            todo.append(("%g%%" % (100 * rate), w.tau_for_rate(rate)))
        primary_tau = todo[2][1]
    elif name == "C4":
        # "about 25 %" by the paper's definition (shared experts in the denominator) = a third of the routed units
        routed_rate = 0.25 * (w.total_units + w.shared_units) / w.total_units
        primary_tau = w.tau_for_rate(routed_rate)
        todo.append(("25% incl. shared", primary_tau))
    else:  # C5: load-aware thresholds (Sec. 4.3) with the hot expert capped at 1.25 x the balanced share of rows
        cap = int(1.25 * spec.T * spec.K / spec.E)
        base = w.tau_for_rate(0.25)
        primary_tau = w.tau_load_aware(base[spec.lo].contiguous(), cap)
        todo.append(("load-aware (25%% thresholds as the maximum, row cap %d)" % cap, primary_tau))
    cases, _ = w.sweep(todo, K, W)
    for rec in cases[1:]:
        rec["proportionality"] = proportionality(cases[0], rec)
    if name == "C5":
        cases[1]["tau_per_resident_expert"] = [[float(v) for v in primary_tau[e].cpu().numpy()] for e in range(spec.lo, spec.hi)]
    kernels, _ = w.kernel_table(primary_tau, K, W)
    out = {"workload": "%s: T=%d D=%d E=%d F=%d top-%d P=%d%s%s" % (
        spec.name, spec.T, spec.D, spec.E, spec.F, spec.K, spec.P,
        (" + %d shared x %d" % (spec.n_shared, spec.F_sh)) if spec.n_shared else "",
        (" resident experts [%d, %d)" % (spec.lo, spec.hi)) if spec.E_res != spec.E else ""),
        "cases": [{k: v for k, v in c.items() if k != "flops"} for c in cases], "kernels_at_primary": kernels}
    w.close()
    return out


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
                    help="only the layer's forward pass of --workload (no reconstruction / threshold selection / decode / "
                         "router / transformation timings, no other workloads): what the rocprofv3 summaries are taken from")
    ap.add_argument("--no-others", action="store_true", help="skip the C3 / C4 / C5 records")
    ap.add_argument("--rates", default="0,0.25,0.5")
    ap.add_argument("--primary-rate", type=float, default=0.25)
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2508_18376_amd as ds
    from paper_2508_18376_amd.thresholds import offset_bins

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    K, W = args.steps, args.warmup

    w = Workload(args.workload, args.tokens, np, torch, ds, keep_host=True)
    spec, layer, x, logits, stream = w.spec, w.layer, w.x, w.logits, w.stream
    host = w.host
    Fp = w.Fp

    def tau_for(rate):
        tau = w.tau_for_rate(rate)
        if spec.name == "C5" and rate > 0:  # the skewed share is run with the load-aware rule on top
            tau = w.tau_load_aware(tau[spec.lo].contiguous(), int(1.25 * spec.T * spec.K / spec.E))
        return tau

    rates = [float(r) for r in args.rates.split(",")]
    if args.primary_rate not in rates:
        rates.append(args.primary_rate)
    todo = [("%g%%" % (100 * rate), tau_for(rate)) for rate in rates]
    primary_label = "%g%%" % (100 * args.primary_rate)
    sweep, g1_ms = w.sweep(todo, K, W, profile_label=primary_label)
    primary = None
    for rate, rec, (_, tau_dev) in zip(rates, sweep, todo):
        rec["target_drop"] = rate
        if abs(rate - args.primary_rate) < 1e-9:
            primary = dict(rec)
            primary["gemm1_ms"] = g1_ms
            primary["tau_dev"] = tau_dev
            primary["tau_table"] = tau_dev.cpu().numpy()
    kernels, g1_flops = w.kernel_table(primary["tau_dev"], K, W)

    g1_ach = g1_flops / (primary["gemm1_ms"] * 1e-3) / 1e12
    traffic = read_traffic(spec.name) if not args.tokens else None
    roofline = {"kernel": "gemm1_mfma_kernel", "bound": "mfma", "achieved": g1_ach, "peak": BF16_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": g1_ach / BF16_PEAK_TFLOPS, "traffic": traffic,
                "traffic_source": ("profiles/gemm1_mfma_kernel_%s_hbm_traffic.txt (rocprofv3 FETCH_SIZE + WRITE_SIZE of an earlier "
                                   "run of this command; counters are not readable from inside the run)" % spec.name)
                if traffic is not None else None,
                "avg_launch_ms": primary["gemm1_ms"], "flops_per_launch": g1_flops}

    zero = next((r for r in sweep if r["target_drop"] == 0.0), None)
    prop = proportionality(zero, primary) if zero else None

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
        rec_flops = 4.0 * spec.D * Fp * w.total_units
        reconstruction = {"profile_importance_ms": rec_ms, "profile_importance_tflops": rec_flops / (rec_ms * 1e-3) / 1e12,
                          "importance_to_perm_ms": perm_ms, "calibration_tokens": spec.T, "metric": 3}
        log("reconstruction: importance of %d tokens %.3f ms (%.0f TFLOP/s), order %.3f ms"
            % (spec.T, rec_ms, reconstruction["profile_importance_tflops"], perm_ms))

        # threshold selection on the device (Sec. 4.3, Sec. 5.3.3): the steps that feed `tau` every batch
        tau_sel = torch.empty((spec.E, spec.P), dtype=torch.float32, device=dev)
        pairs_sel = torch.empty((spec.E,), dtype=torch.int32, device=dev)
        tau_max_dev = primary["tau_dev"][spec.lo].contiguous()
        cap_rows = int(1.25 * spec.T * spec.K / spec.E)
        sel_ms = ev_ms(lambda: ds.moe_select_thresholds(layer.ctx, logits, spec.T, tau_max_dev, 1, cap_rows, tau_sel, pairs_sel,
                                                        layer.workspace, stream), max(10, K))
        stats_sel = torch.empty((2,), dtype=torch.int32, device=dev)
        rate_ms = ev_ms(lambda: ds.moe_thresholds_for_drop_rate(layer.ctx, logits, spec.T, args.primary_rate, offset_bins(spec.P),
                                                                tau_sel, stats_sel, layer.workspace, stream), max(10, K))
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
        ds.moe_pack_router(layer.ctx, w.up(wg_host), router_packed, stream)
        lg_out = torch.empty((spec.T, spec.E), dtype=torch.float32, device=dev)
        router_ms = ev_ms(lambda: ds.moe_router_logits(layer.ctx, router_packed, x, spec.T, lg_out, stream), max(10, K))
        routed_ms = ev_ms(lambda: ds.moe_dualsparse_forward_routed(layer.ctx, layer.packed, router_packed, x, primary["tau_dev"],
                                                                   spec.T, w.y, None, layer.workspace, stream), max(5, K // 2))
        router_bytes = spec.T * spec.D * 2 + spec.T * spec.E * 4
        router = {"router_logits_ms": router_ms, "GBps": router_bytes / (router_ms * 1e-3) / 1e9,
                  "forward_routed_ms": routed_ms}
        log("router x W_g: %.4f ms (%.0f GB/s of x); layer driven by those logits (another routing, same tau table) %.3f ms"
            % (router_ms, router["GBps"], routed_ms))
        del lg_out
        w_dev = {k: w.up(host[k]) for k in ("w1", "w3", "w2")}
        w_out = {k: torch.empty_like(v) for k, v in w_dev.items()}
        wg_dev, wg_out = w.up(wg_host), torch.empty((spec.D, spec.E * spec.P), dtype=torch.bfloat16, device=dev)
        perm_dev = w.up(host["perm"])
        tr_ms = ev_ms(lambda: ds.moe_transform_complete(layer.ctx, wg_dev, w_dev["w1"], w_dev["w3"], w_dev["w2"], perm_dev, wg_out,
                                                        w_out["w1"], w_out["w3"], w_out["w2"], layer.workspace, stream), 2)
        w_bytes = sum(v.numel() * 2 for v in w_dev.values())
        transform = {"transform_complete_ms": tr_ms, "GBps": 2 * w_bytes / (tr_ms * 1e-3) / 1e9}
        log("complete transformation of %.2f GB of weights: %.2f ms (%.0f GB/s read + write)" % (w_bytes / 1e9, tr_ms, transform["GBps"]))
        del w_dev, w_out

        # decode-sized batches of the same layer (weight streaming regime): the first T tokens of the batch
        w_unit_bytes = 3 * spec.D * Fp * 2
        for Td in (16, 64, 256):
            if Td > spec.T:
                continue
            xd, ld = x[:Td].contiguous(), logits[:Td].contiguous()
            tau_d = w.tau_for_rate(args.primary_rate, T=Td)
            w.kept_units(tau_d, T=Td, logits=ld)
            gc = w.r_gc.cpu().numpy()
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
                           "frac_hbm_peak": wbytes / (ms_d * 1e-3) / 1e9 / HBM_PEAK_GBS})
            log("decode T=%d: %.3f ms/step, weights of %d active sub-experts %.2f GB -> %.0f GB/s (%.0f %% of 8 TB/s)"
                % (Td, ms_d, active, wbytes / 1e9, decode[-1]["GBps"], 100 * decode[-1]["frac_hbm_peak"]))

    # CPU oracle leg: the same layer and thresholds on a seeded token sample, all host cores
    cpu = None
    check = None
    if not args.no_cpu:
        import oracle
        S = args.sample or {"C2": 1536, "C3": 8192, "C4": 6144, "C5": 2048}[spec.name]  # about 10 s of oracle time each
        S = min(S, spec.T)
        tok = np.sort(np.random.default_rng(12345).choice(spec.T, size=S, replace=False)).astype(np.int32)
        tau_host = primary["tau_table"]
        t0 = time.time()
        y_ref = oracle.forward(host["x"], host["logits"], host["w1"], host["w3"], host["w2"], tau_host, spec.K,
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
        # the thresholds sit on the device's grid, not in a gap between scores: tokens whose fp32 and fp64
        # keep decisions could differ (|n - tau| <= 1e-6) are left out of the comparison, and counted
        margin = oracle.route(host["logits"], spec.K, spec.P, tau_host, spec.lo, spec.hi)
        n64 = margin.n
        near = np.zeros(spec.T, dtype=bool)
        for p in range(spec.P):
            near |= (np.abs(n64 - tau_host[margin.idx, p].astype(np.float64)) <= 1e-6).any(axis=1)
        ok_rows = ~near[tok]
        # the timed output (bf16) and, from the same packed weights, the fp32 output that carries no output rounding
        w.run(primary["tau_dev"], 1)
        ctx32 = ds.dsmoe_create(d_model=spec.D, d_ff=spec.F, n_experts=spec.E, top_k=spec.K, n_part=spec.P, max_tokens=spec.T,
                                dtype=1, n_shared=spec.n_shared, d_ff_shared=spec.F_sh, expert_lo=spec.lo, expert_hi=spec.hi,
                                y_fp32=1)
        y32 = torch.empty((spec.T, spec.D), dtype=torch.float32, device=dev)
        ds.moe_dualsparse_forward(ctx32, layer.packed, x, logits, primary["tau_dev"], spec.T, y32, layer.workspace, stream)
        torch.cuda.synchronize()
        ds.dsmoe_destroy(ctx32)
        sel = torch.from_numpy(tok.astype(np.int64)).to(dev)
        a16 = w.y[sel].to(torch.float32).cpu().numpy().astype(np.float64)[ok_rows]
        a32 = y32[sel].cpu().numpy().astype(np.float64)[ok_rows]
        ref = y_ref[ok_rows]
        rms = float(np.sqrt(np.mean(ref ** 2)))
        e16, e32 = np.abs(a16 - ref), np.abs(a32 - ref)
        beyond16 = e16 - 2.0 ** -8 * np.abs(ref)  # the bf16 output format costs up to 2^-8 |y| by itself
        check = {"elements": int(ref.size), "tolerance": 2e-2, "tokens_left_out_near_a_threshold": int((~ok_rows).sum()),
                 "fp32_output": {"max_err_over_rms": float(e32.max() / rms), "rms_err_over_rms": float(np.sqrt(np.mean(e32 ** 2)) / rms),
                                 "elements_beyond_tolerance": int((e32 > 2e-2 * rms).sum())},
                 "bf16_output": {"max_err_over_rms": float(e16.max() / rms),
                                 "max_err_beyond_output_rounding_over_rms": float(beyond16.max() / rms),
                                 "elements_beyond_tolerance_plus_output_rounding": int((beyond16 > 2e-2 * rms).sum())}}
        log("oracle: %.2f tokens/s on %d threads; GPU vs oracle on the sample: fp32 output max |err| %.4f x RMS (bar 0.02, %d "
            "elements over); bf16 output %.4f x RMS, %.4f x RMS beyond its own rounding" % (
                cpu["value"], cpu["cores"], check["fp32_output"]["max_err_over_rms"],
                check["fp32_output"]["elements_beyond_tolerance"], check["bf16_output"]["max_err_over_rms"],
                check["bf16_output"]["max_err_beyond_output_rounding_over_rms"]))

    workload_line = "%s: T=%d D=%d E=%d F=%d top-%d P=%d%s, tau for ~%d%% unit drop (realised %.1f%%)" % (
        spec.name, spec.T, spec.D, spec.E, spec.F, spec.K, spec.P,
        (" + %d shared x %d" % (spec.n_shared, spec.F_sh)) if spec.n_shared else "",
        round(100 * args.primary_rate), 100 * primary["drop_rate"])
    resident = [spec.lo, spec.hi]
    w.close()
    del w, layer, x, logits, host

    workloads = {}
    if not args.core_only and not args.no_others and not args.tokens and args.workload == "C2":
        for name in ("C3", "C4", "C5"):
            workloads[name] = other_workload(name, np, torch, ds, K, W)

    def strip(r):
        return {k: v for k, v in r.items() if k not in ("flops", "tau_dev", "tau_table", "gemm1_ms")}

    out = {
        "metric": "MoE-layer tokens/s + MFMA TFLOP/s vs bf16 peak at 0/25/50% drop",
        "value": primary["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": primary["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": workload_line, "resident_experts": resident, "tokens": spec.T,
                   "thresholds": "chosen on the device by moe_thresholds_for_drop_rate from the batch's scores",
                   "timing": "every case: median of 3 passes of `steps` timed steps after `warmup` steps, the cases of a sweep "
                             "interleaved pass by pass"},
        "tflops": primary["tflops"], "frac_bf16_peak": primary["frac_bf16_peak"],
        "sweep": [strip(r) for r in sweep], "proportionality": prop, "kernels": kernels,
        "kernels_note": "HIP-event intervals around each launch of a separate timing pass: every entry carries about 4 us of "
                        "event-to-event gap (an empty interval reads 4-5 us); kernel durations proper are in profiles/",
        "workloads": workloads,
        "reconstruction": reconstruction, "threshold_selection": selection, "decode": decode, "router": router,
        "complete_transformation": transform,
        "roofline": roofline, "cpu_baseline": cpu, "check": check,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
