#!/usr/bin/env python3
"""Benchmark of the correlation-lookup hot path on ONE MI355X.

A step = one image pair = one corr_pyramid_build (feature re-layout + pooled
levels) followed by `--lookups` corr_sample calls (binning pass, block
contraction + bilinear epilogue for every level) on different coordinates.
Inputs are resident in HBM before the timed region.  Prints one JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E
PEAK_FP32_MFMA_TFS = 157.3    # MI355X dense fp32 MFMA


def kernel_source_sha() -> str:
    """sha256 over the library's kernel sources: ties a counter summary to the code it measured."""
    from paper_2505_16942_amd.profile_summary import kernel_source_sha as sha
    return sha()


def bench_backward(args, cb, synth, torch, np) -> int:
    """The gradient entry point: `value` = tap gradients (queries x L x 81) taken back per second."""
    dev = torch.device("cuda:0")
    cfg = synth.config(args.config)
    B, H, W, D, L, r = cfg["B"], cfg["H"], cfg["W"], cfg["D"], cfg["L"], cfg["r"]
    K = 2 * r + 1
    N = H * W
    f1, f2 = synth.features(cfg)
    c = synth.coords(cfg, 0)
    t1, t2, tc = (torch.from_numpy(a).to(dev) for a in (f1, f2, c))
    gen = torch.Generator(device=dev)
    gen.manual_seed(cfg["seed"])
    d_out = torch.randn((B, L * K * K, H, W), device=dev, generator=gen)
    pyr = cb.corr_pyramid_build(t1, t2, L=L, reps=cb.CORR_REP_F32)
    ws = torch.empty(cb.corr_backward_workspace_bytes(B, H, W, D, L) // 4, device=dev)
    g1 = torch.empty_like(t1)
    g2 = torch.empty_like(t1)
    form = cb.CORR_BACKWARD_QUERIES if args.backward_form == "queries" else cb.CORR_BACKWARD_ITEMS
    cb.corr_debug_set_backward_form(form)
    for _ in range(max(args.warmup, 1)):
        cb.corr_sample_backward(pyr, tc, d_out, r=r, d_fmap1=g1, d_fmap2=g2, workspace=ws)
    torch.cuda.synchronize()
    tb = time.perf_counter()
    for _ in range(args.steps):
        cb.corr_sample_backward(pyr, tc, d_out, r=r, d_fmap1=g1, d_fmap2=g2, workspace=ws)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - tb) / args.steps
    cb.corr_debug_set_backward_form(cb.CORR_BACKWARD_ITEMS)
    taps = B * N * L * K * K
    npyr = sum((H >> l) * (W >> l) for l in range(L))
    # algorithmic HBM bytes: d_out, fmap1 and every pyramid pixel (fp32) read once, both gradients written once
    bytes_alg = B * (taps // B * 4 + N * D * 4 + npyr * D * 4 + N * 8 + 2 * N * D * 4)
    gbs = bytes_alg / dt / 1e9
    # the item form's two dense contractions: every query against every point of its cell's window, per level
    win = sum((max(16 >> l, 1) + K) * (max(8 >> l, 1) + K) for l in range(L))
    flops_dense = 4.0 * B * N * win * D
    flops_footprint = 4.0 * B * N * L * (K + 1) ** 2 * D       # what the gradient needs at the least
    tfs = flops_dense / dt / 1e12
    if form == cb.CORR_BACKWARD_ITEMS:
        roof = {"bound": "mfma", "achieved": round(tfs, 2), "peak": PEAK_FP32_MFMA_TFS, "unit": "TFLOP/s",
                "frac": round(tfs / PEAK_FP32_MFMA_TFS, 4), "traffic": None,
                "kernel": "bwd_item_kernel (per work item and level: G^T x f2 rows and G x f1 rows on fp32 MFMA, "
                          "window rows of d f2 out through float atomics); the time is the whole call's",
                "flops_per_call": flops_dense, "footprint_flops_per_call": flops_footprint,
                "hbm": {"achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(gbs / PEAK_HBM_GBS, 4),
                        "algorithmic_bytes_per_call": bytes_alg},
                "note": "flops = 4 * queries * window points of the cell (%d over the levels) * D, unpadded; "
                        "peak = dense fp32 MFMA" % win}
    else:
        atomics = float(B * N * L * (K + 1) ** 2 * D)
        roof = {"bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": round(gbs / PEAK_HBM_GBS, 4), "traffic": None,
                "kernel": "bwd_query_kernel (one wave per query, float atomics into the level gradients)",
                "algorithmic_bytes_per_launch": bytes_alg,
                "note": "the one-wave-per-query form: its time is the atomics', at most %.3g of them per call, "
                        "%.0f G/s here" % (atomics, atomics / dt / 1e9)}
    result = {
        "metric": "correlation lookup gradient, tap gradients/s (queries x L x 81 taps)", "value": taps / dt,
        "unit": "tap gradients/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: B=%d fmap [%d,%d,%d,%d] L=%d r=%d; step = one corr_sample_backward (%s form)"
                               % (args.config, B, B, D, H, W, L, r, args.backward_form), "seed": cfg["seed"]},
        "roofline": roof,
    }
    pyr.destroy()
    print(json.dumps(result))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", default="8k", choices=["tiny", "1080p", "4k", "8k", "voronoi"])
    ap.add_argument("--lookups", type=int, default=12, help="corr_sample calls per pyramid build")
    ap.add_argument("--prec", default="bf16x3", choices=["bf16x3", "bf16"])
    ap.add_argument("--out-layout", default="nchw", choices=["nchw", "nhwc"],
                    help="layout of out: nchw is the headline (what the paper's kernel writes); nhwc is the "
                         "library's channels-last option")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-4k", action="store_true",
                    help="skip the short 4k measurement (12 recurrent lookups per pair) that an 8k run appends")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU work for the oracle sample")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run the library's plain copy kernel on 1 GiB (3 launches) so that a counter run "
                         "sees a kernel of known HBM traffic")
    ap.add_argument("--print-source-sha", action="store_true", help="print the kernel-source hash and exit")
    ap.add_argument("--backward", action="store_true",
                    help="time the gradient of the lookup (corr_sample_backward) instead: a step = one call on the "
                         "workload's first coordinates; its own JSON line")
    ap.add_argument("--backward-form", default="items", choices=["items", "queries"],
                    help="with --backward: the work-item form on the matrix cores (default) or the earlier one-wave-per-query form")
    ap.add_argument("--compare-modes", action="store_true",
                    help="additionally time the on-demand and full-volume reference modes (one lookup each)")
    args = ap.parse_args()
    if args.print_source_sha:
        print(kernel_source_sha())
        return 0
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2505_16942_amd import binding as cb
    from paper_2505_16942_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1
    cb.load_library()
    if args.backward:
        return bench_backward(args, cb, synth, torch, np)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cfg = synth.config(args.config)
    B, H, W, D, L, r = cfg["B"], cfg["H"], cfg["W"], cfg["D"], cfg["L"], cfg["r"]
    K = 2 * r + 1
    N = H * W
    nl = args.lookups
    prec = cb.CORR_PREC_BF16X3 if args.prec == "bf16x3" else cb.CORR_PREC_BF16
    terms = 3 if args.prec == "bf16x3" else 1
    layout = cb.CORR_OUT_NHWC if args.out_layout == "nhwc" else cb.CORR_OUT_NCHW
    rep = cb.CORR_REP_SPLIT if terms == 3 else cb.CORR_REP_BF16     # bf16 mode: hi parts alone, half the bytes

    t0 = time.time()
    f1, f2 = synth.features(cfg)
    coords_h = [synth.coords(cfg, t) for t in range(nl)]
    gen_s = time.time() - t0
    t1, t2 = torch.from_numpy(f1).to(dev), torch.from_numpy(f2).to(dev)
    tcs = [torch.from_numpy(c).to(dev) for c in coords_h]
    out = torch.empty((B, H, W, L * K * K) if layout == cb.CORR_OUT_NHWC else (B, L * K * K, H, W),
                      dtype=torch.float32, device=dev)
    torch.cuda.synchronize()
    torch.cuda.reset_peak_memory_stats()

    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)      # 1 GiB read + 1 GiB written per launch
        dst = torch.empty_like(src)
        for _ in range(3):
            cb.corr_copy_f32(dst, src)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()
        torch.cuda.reset_peak_memory_stats()

    pyr = cb.corr_pyramid_build(t1, t2, L=L, reps=rep)

    def step():
        cb.corr_pyramid_build(t1, t2, L=L, reps=rep, pyramid=pyr)
        for tc in tcs:
            cb.corr_sample(t1, pyr, tc, r=r, out=out, prec=prec, layout=layout)

    # untimed: per-lookup work counters of the binning pass (they depend on the coordinates)
    cb.corr_pyramid_build(t1, t2, L=L, reps=rep, pyramid=pyr)
    stats = []
    for tc in tcs:
        cb.corr_sample(t1, pyr, tc, r=r, out=out, prec=prec, layout=layout)
        stats.append(cb.corr_last_block_stats(pyr, r))
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # the headline: K steps between synchronisations, the library's profiling hook off
    cb.corr_profile_enable(False)
    torch.cuda.synchronize()
    tb = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    te = time.perf_counter()

    # per-kernel durations: a separate pass over the same steps with HIP events around each kernel on the
    # launch stream (the library records them); the hook keeps PROF_CAP lookups, so the pass is sized to fit
    PROF_CAP = 256
    prof_steps = max(1, min(args.steps, PROF_CAP // nl))
    cb.corr_profile_enable(True)
    for _ in range(prof_steps):
        step()
    torch.cuda.synchronize()
    prof = cb.corr_profile_read()
    cb.corr_profile_enable(False)
    if prof.get("dropped", 0):
        print("bench.py: warning: %d profiled lookups were dropped (cap %d)" % (prof["dropped"], PROF_CAP), file=sys.stderr)

    ms_per_step = (te - tb) * 1e3 / args.steps
    lookups_per_call = B * N * L * K * K
    value = lookups_per_call * nl * args.steps / (te - tb)

    # separate timings (untimed region): build alone, lookups alone
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    reps_t = 5
    ev[0].record()
    for _ in range(reps_t):
        cb.corr_pyramid_build(t1, t2, L=L, reps=rep, pyramid=pyr)
    ev[1].record()
    for _ in range(reps_t):
        for tc in tcs:
            cb.corr_sample(t1, pyr, tc, r=r, out=out, prec=prec, layout=layout)
    ev[2].record()
    torch.cuda.synchronize()
    build_ms = ev[0].elapsed_time(ev[1]) / reps_t
    lookup_ms = ev[1].elapsed_time(ev[2]) / (reps_t * nl)

    # ---- roofline of the dominant kernel: the block kernel (contraction + epilogue, all levels)
    nprof = max(prof["lookups"], 1)
    blk_ms = prof["block_ms"] / nprof
    bin_ms = prof["binning_ms"] / nprof
    used_pq = float(np.mean([s["used_point_queries"] for s in stats]))
    mma_pq = float(np.mean([s["mma_point_queries"] for s in stats]))
    # flops the method defines: one D-long dot product per (window point, real query) pair; the bf16x3
    # mode runs each as three bf16 MFMA terms, which is more machine work, not more useful work
    flops_1 = 2.0 * D * used_pq
    flops_run = flops_1 * terms
    npyr = sum((H >> l) * (W >> l) for l in range(L))
    # algorithmic HBM bytes of one launch: fmap1 and every pyramid pixel once (bf16 hi+lo = 4 B per
    # element; bf16 mode on hi-only records 2 B), coords, the sorted query list, `out` once
    feat_b = 4 if terms == 3 else 2
    bytes_alg = B * (N * D * feat_b + npyr * D * feat_b + N * 8 + N * 4 + N * L * K * K * 4)
    hbm_floor_ms = bytes_alg / (PEAK_HBM_GBS * 1e9) * 1e3
    mfma_floor_ms = flops_run / (PEAK_BF16_TFLOPS * 1e12) * 1e3
    hbm_gbs = bytes_alg / (blk_ms * 1e-3) / 1e9
    tf_run = flops_run / (blk_ms * 1e-3) / 1e12
    tf_1 = flops_1 / (blk_ms * 1e-3) / 1e12
    if hbm_floor_ms >= mfma_floor_ms:       # the binding roofline is the one with the larger time floor
        roofline = {"bound": "hbm", "achieved": round(hbm_gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": round(hbm_gbs / PEAK_HBM_GBS, 4)}
    else:
        roofline = {"bound": "mfma", "achieved": round(tf_run, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(tf_run / PEAK_BF16_TFLOPS, 4)}
    roofline.update({
        "traffic": None, "traffic_source": None,
        "kernel": "block_kernel (contraction + bilinear epilogue, all %d levels)" % L,
        "avg_launch_ms": round(blk_ms, 4), "launches_timed": int(prof["lookups"]),
        "algorithmic_bytes_per_launch": bytes_alg,
        "floors_ms": {"hbm": round(hbm_floor_ms, 4), "mfma_as_run": round(mfma_floor_ms, 4)},
        "hbm": {"achieved_GBs": round(hbm_gbs, 1), "frac": round(hbm_gbs / PEAK_HBM_GBS, 4)},
        "mfma": {"flops_method_1term": flops_1, "flops_as_run_%dterm" % terms: flops_run,
                 "TFLOPs_1term": round(tf_1, 2), "frac_1term": round(tf_1 / PEAK_BF16_TFLOPS, 4),
                 "TFLOPs_as_run": round(tf_run, 2), "frac_as_run": round(tf_run / PEAK_BF16_TFLOPS, 4),
                 "issued_over_counted": round(mma_pq / max(used_pq, 1.0), 4),
                 "counted": "2*D*window points*real queries summed over levels; as_run multiplies by the %d bf16 "
                            "terms of this precision; issued adds padding rows and empty query slots" % terms},
    })

    # HBM traffic of the block kernel is not measured by this run (it needs hardware counters).  A committed
    # counter summary is quoted only if it says it was taken on exactly the kernel sources in this tree.
    traffic_file = os.path.join(ROOT, "profiles", "block_kernel_%s_hbm_traffic.txt" % args.config)
    if terms == 3 and args.out_layout == "nchw" and os.path.exists(traffic_file):
        fields = {}
        for line in open(traffic_file):
            if ":" in line and not line.startswith("#"):
                k, v = line.split(":", 1)
                fields[k.strip()] = v.strip()
        if fields.get("kernel_source_sha256", "")[:16] == kernel_source_sha()[:16] and "traffic_bytes_per_launch" in fields:
            roofline["traffic"] = float(fields["traffic_bytes_per_launch"])
            roofline["traffic_source"] = {"file": os.path.relpath(traffic_file, ROOT), "measured": fields.get("date", "?"),
                                          "kernel_source_sha256": fields["kernel_source_sha256"][:16],
                                          "note": "rocprofv3 FETCH_SIZE/WRITE_SIZE runs of this command, not this run"}
        else:
            roofline["traffic_source"] = "committed counter summary is for other kernel sources; not quoted"

    peak_bytes = int(torch.cuda.max_memory_allocated()) + pyr.bytes()
    result = {
        "metric": "correlation lookups/s (queries x L x 81 taps)", "value": value, "unit": "lookups/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16x3->f32" if terms == 3 else "bf16->f32", "data": "synthetic",
        "config": {"workload": "%s: B=%d fmap [%d,%d,%d,%d] L=%d r=%d; step = 1 pyramid build + %d lookups"
                               % (args.config, B, B, D, H, W, L, r, nl),
                   "seed": cfg["seed"], "lookups_per_build": nl, "lookups_per_call": lookups_per_call,
                   "out_layout": args.out_layout},
        "roofline": roofline,
        "breakdown_ms": {"pyramid_build": round(build_ms, 4), "one_lookup": round(lookup_ms, 4),
                         "binning_pass": round(bin_ms, 4),
                         "block_kernel": round(blk_ms, 4)},
        "lookup_only_lookups_per_s": lookups_per_call / (lookup_ms * 1e-3),
        "peak_device_bytes": peak_bytes, "library_bytes": pyr.bytes(),
        "full_volume_bytes": cb.corr_full_volume_bytes(B, H, W, L),
        "binning": {"items": float(np.mean([s["items"] for s in stats])),
                    "null_query_levels": float(np.mean([s["null_query_levels"] for s in stats])),
                    "window_points_per_query_level": float(np.mean(
                        [s["used_point_queries"] / max(s["query_levels"] - s["null_query_levels"], 1) for s in stats]))},
        "input_generation_s": round(gen_s, 1),
    }

    if args.compare_modes:
        # one lookup in each reference mode on the same inputs (full volume only if it fits)
        pyr2 = cb.corr_pyramid_build(t1, t2, L=L, reps=cb.CORR_REP_F32)
        modes = {}
        for name, mode in (("ondemand", cb.CORR_MODE_ONDEMAND), ("fullvolume", cb.CORR_MODE_FULLVOLUME)):
            try:
                cb.corr_sample(t1, pyr2, tcs[0], r=r, out=out, mode=mode, layout=layout)      # full volume: builds the volume
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                cb.corr_sample(t1, pyr2, tcs[0], r=r, out=out, mode=mode, layout=layout)
                e1.record()
                torch.cuda.synchronize()
                ms = e0.elapsed_time(e1)
                modes[name] = {"one_lookup_ms": round(ms, 3), "lookups_per_s": lookups_per_call / (ms * 1e-3),
                               "library_bytes": pyr2.bytes()}
            except cb.CorrError as err:
                modes[name] = {"status": str(err), "needs_bytes": cb.corr_full_volume_bytes(B, H, W, L)}
        modes["block"] = {"one_lookup_ms": round(lookup_ms, 3), "lookups_per_s": lookups_per_call / (lookup_ms * 1e-3),
                          "library_bytes": pyr.bytes()}
        result["modes"] = modes
        pyr2.destroy()

    if not args.no_cpu_baseline:
        from oracle import corr_oracle
        rng = np.random.default_rng(cfg["seed"])
        c0 = coords_h[0]
        tq = time.perf_counter()
        corr_oracle.lookup_points(f1, f2, c0, np.zeros(1, np.int64), L=L, r=r)
        prep_s = time.perf_counter() - tq          # the oracle's own per-pair preprocessing
        nq_cal = min(B * N, 20000)
        def sample_idx(nq):
            qs = rng.choice(B * N, size=min(nq, B * N), replace=False)
            b, p = qs // N, qs % N
            ch = np.arange(L * K * K)
            return ((b[:, None] * (L * K * K) + ch[None, :]) * N + p[:, None]).reshape(-1).astype(np.int64)
        idx = sample_idx(nq_cal)
        tq = time.perf_counter()
        corr_oracle.lookup_points(f1, f2, c0, idx, L=L, r=r)
        cal_s = max(time.perf_counter() - tq - prep_s, 0.05)
        nq = int(min(B * N, max(nq_cal, nq_cal * args.cpu_seconds / cal_s)))
        idx = sample_idx(nq)
        tq = time.perf_counter()
        vals = corr_oracle.lookup_points(f1, f2, c0, idx, L=L, r=r)
        tot_s = time.perf_counter() - tq
        work_s = max(tot_s - prep_s, 1e-6)
        # the same sample on the GPU result of lookup 0: parity of what was timed
        cb.corr_sample(t1, pyr, tcs[0], r=r, out=out, prec=prec, layout=layout)
        torch.cuda.synchronize()
        out_nchw = out.permute(0, 3, 1, 2) if layout == cb.CORR_OUT_NHWC else out     # indices are NCHW
        got = out_nchw.reshape(-1)[torch.from_numpy(idx).to(dev)].cpu().numpy().astype(np.float64)
        maxc = float(np.abs(vals).max())
        result["cpu_baseline"] = {
            "value": idx.size / work_s, "unit": "lookups/s", "cores": corr_oracle.threads(), "kind": "oracle",
            "sample": "%d random queries x all %d taps of lookup 0 (%d lookups), fp64 per-tap oracle; "
                      "%.1f s of tap work, its per-pair preprocessing (%.1f s) excluded"
                      % (nq, L * K * K, idx.size, work_s, prep_s),
            # like for like with `value` (one preprocessing per pair, then every lookup of the step),
            # extrapolated from the sample's tap rate
            "whole_step_value": lookups_per_call * nl / (prep_s + lookups_per_call * nl * work_s / idx.size),
            "whole_step_note": "lookups of one step / (measured per-pair preprocessing + the step's lookups at the "
                               "sampled tap rate)"}
        result["parity_on_sample"] = {"max_abs_err": float(np.abs(got - vals).max()), "max_abs_C": maxc,
                                      "bound": (1e-4 if terms == 3 else 2e-2) * maxc}
    pyr.destroy()
    if args.config == "8k" and not args.no_4k:
        # the metric is quoted at 4K and 8K scale: the same step on the 4k workload (12 lookups of one
        # pair whose flow does a per-pixel random walk), same precision and layout, reported beside the headline
        del t1, t2, tcs, out
        torch.cuda.empty_cache()
        c4 = synth.config("4k")
        g1, g2 = synth.features(c4)
        u1, u2 = torch.from_numpy(g1).to(dev), torch.from_numpy(g2).to(dev)
        ucs = [torch.from_numpy(synth.coords(c4, t)).to(dev) for t in range(12)]
        B4, H4, W4, L4 = c4["B"], c4["H"], c4["W"], c4["L"]
        o4 = torch.empty((B4, H4, W4, L4 * K * K) if layout == cb.CORR_OUT_NHWC else (B4, L4 * K * K, H4, W4),
                         dtype=torch.float32, device=dev)
        p4 = cb.corr_pyramid_build(u1, u2, L=L4, reps=rep)

        def step4():
            cb.corr_pyramid_build(u1, u2, L=L4, reps=rep, pyramid=p4)
            for tc in ucs:
                cb.corr_sample(u1, p4, tc, r=r, out=o4, prec=prec, layout=layout)

        for _ in range(args.warmup + 1):
            step4()
        torch.cuda.synchronize()
        t4 = time.perf_counter()
        for _ in range(args.steps):
            step4()
        torch.cuda.synchronize()
        dt4 = time.perf_counter() - t4
        result["at_4k"] = {"workload": "4k: B=1 fmap [1,256,270,480] L=4 r=4; step = 1 pyramid build + 12 lookups",
                           "value": B4 * H4 * W4 * L4 * K * K * 12 * args.steps / dt4, "unit": "lookups/s",
                           "ms_per_step": dt4 * 1e3 / args.steps, "steps": args.steps}
        p4.destroy()
        # and the gradient of the lookup on the same 4k pair (its own line: bench.py --backward): a few calls
        pg = cb.corr_pyramid_build(u1, u2, L=L4, reps=cb.CORR_REP_F32)
        gen = torch.Generator(device=dev)
        gen.manual_seed(c4["seed"])
        d_out = torch.randn((B4, L4 * K * K, H4, W4), device=dev, generator=gen)
        wsb = torch.empty(cb.corr_backward_workspace_bytes(B4, H4, W4, c4["D"], L4) // 4, device=dev)
        q1, q2 = torch.empty_like(u1), torch.empty_like(u1)
        for _ in range(2):
            cb.corr_sample_backward(pg, ucs[0], d_out, r=r, d_fmap1=q1, d_fmap2=q2, workspace=wsb)
        torch.cuda.synchronize()
        tb = time.perf_counter()
        for _ in range(args.steps):
            cb.corr_sample_backward(pg, ucs[0], d_out, r=r, d_fmap1=q1, d_fmap2=q2, workspace=wsb)
        torch.cuda.synchronize()
        dtb = (time.perf_counter() - tb) / args.steps
        win = sum((max(16 >> l, 1) + K) * (max(8 >> l, 1) + K) for l in range(L4))
        tfs = 4.0 * B4 * H4 * W4 * win * c4["D"] / dtb / 1e12
        result["backward_at_4k"] = {"workload": "4k, one corr_sample_backward per step (fp32, work items on fp32 MFMA)",
                                    "value": B4 * H4 * W4 * L4 * K * K / dtb, "unit": "tap gradients/s",
                                    "ms_per_step": dtb * 1e3, "steps": args.steps,
                                    "roofline": {"bound": "mfma", "achieved": round(tfs, 2), "peak": PEAK_FP32_MFMA_TFS,
                                                 "unit": "TFLOP/s", "frac": round(tfs / PEAK_FP32_MFMA_TFS, 4)}}
        pg.destroy()
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
