#!/usr/bin/env python3
"""Benchmark of the two-stage DDCCANet hot path on one MI355X.

One "step" = the whole path on one synthetic workload, inputs already in HBM:
  learn the stage-1 filters -> learn the stage-2 filters from the same inputs (the stage-1 maps of the training
  set are convolved batch by batch into library scratch and accumulated at once, never held as a whole)
  -> extract_features for all images (stage-1 conv, stage-2 conv with the maps of a batch materialised,
  hashing + block histograms).
Prints ONE JSON line.  `value` is on the headline workload (default: large_scale, the largest single-GPU
configuration); `other_workloads` carries images/s and the per-kernel figures of the other configurations measured
in the same run; `roofline` is the dominant kernel (patch-Gram, fp32 MFMA) timed with HIP events on the library's
stream; `cpu_baseline` is the CPU oracle on a bounded sample of the headline workload.
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_MFMA_FP32_TFLOPS = 157.3      # MI355X dense fp32 matrix peak
PEAK_MFMA_BF16_TFLOPS = 2500.0     # MI355X dense bf16 matrix peak
PEAK_HBM_GBS = 8000.0              # MI355X HBM3E
ALL_WORKLOADS = ["large_scale", "stress", "object", "small_face", "tiny"]
CPU_SAMPLE_IMAGES = {"tiny": 40, "small_face": 400, "object": 128, "large_scale": 257, "stress": 16}


def algorithmic_work(wl, M, feat_bytes=2):
    """Algorithmic flops / bytes per step for each kernel (both stages, both views)."""
    D, P = wl.D, wl.h * wl.w
    L1, L2, C = wl.L1, wl.L2, wl.n_classes
    by, bx = wl.blocks
    A, bins = by * bx, 1 << wl.L2
    per_patch = 2.0 * (2 * D * D + D)                 # two symmetric blocks + one full block
    gram_main = per_patch * (M * P + M * L1 * P)
    gram_class = 2.0 * D * D * P * ((C * 1 + 1) + (C * L1 + L1))   # cross block of class-sum / total images
    # conv: read 4 B, write 4L B per input pixel; stage 1 runs in fit (the samples and the C + 1 sum images of
    # the second learning stage) and again in extract
    conv_bytes = 2 * ((2 * M + C + 1) * P * (4 + 4 * L1)) + 2 * M * L1 * P * (4 + 4 * L2)
    conv_flops = 2 * ((2 * M + C + 1) * P * 2 * D * L1) + 2 * M * L1 * P * 2 * D * L2
    hist_bytes = 2 * M * L1 * (L2 * P * 4 + A * bins * feat_bytes)
    class_bytes = 2 * 4 * (M * P + M * P)            # the inputs of both views, read once per learning stage
    return {
        "gram_flops": gram_main, "gram_cross_flops": gram_class,
        "conv_bytes": conv_bytes, "conv_flops": conv_flops, "hist_bytes": hist_bytes,
        "class_sum_bytes": class_bytes,
    }


def measured_traffic(workload, kernel_regex):
    """HBM bytes per launch (read + write) of the kernels whose name matches `kernel_regex`, from the
    rocprofv3 --pmc passes summarised in profiles/traffic.json (FETCH_SIZE / WRITE_SIZE scaled by a plain
    copy of known size); None when no profile of this workload is committed."""
    import re
    path = os.path.join(ROOT, "profiles", "traffic.json")
    if not os.path.exists(path):
        return None
    with open(path) as f:
        data = json.load(f).get(workload)
    if not data:
        return None
    tot_bytes, tot_launches = 0.0, 0
    for name, v in data.items():
        if re.match(kernel_regex, name) and "read_mib_per_launch" in v:
            tot_bytes += v["launches"] * (v["read_mib_per_launch"] + v["write_mib_per_launch"]) * 1048576.0
            tot_launches += v["launches"]
    return tot_bytes / tot_launches if tot_launches else None


def run_cpu_baseline(wl, budget_images):
    """Time the fp64 CPU oracle (whole path) on a bounded class-balanced sample."""
    from oracle import ddcca_oracle as oracle
    from paper_2209_13027_amd.workloads import make_views
    per_class = max(1, budget_images // wl.n_classes)
    v1, v2, cls = make_views(wl, max_per_class=per_class)
    t0 = time.perf_counter()
    oracle.two_stage(v1, v2, cls, wl.n_classes, wl.k, wl.L1, wl.L2, wl.block)
    dt = time.perf_counter() - t0
    n = int(v1.shape[0])
    return {
        "value": n / dt, "unit": "images/s", "cores": oracle.num_threads(), "kind": "oracle",
        "sample": f"{n} of {wl.M} images of {wl.name} ({per_class} per class), whole path (learn both stages + "
                  f"extract), fp64, {dt:.1f} s",
    }


def measure(name, args, K, W, detail):
    """All figures of one workload.  detail: the comparison legs too (phases, fused / bf16x3 extraction, the cost of
    the timing events)."""
    import torch
    from paper_2209_13027_amd import pipeline
    from paper_2209_13027_amd.binding import (Context, OPT_CONV_ARITH, CONV_BF16X3, CONV_FP32, CONV_AUTO,
                                              OPT_GRAM_ARITH, GRAM_FP32, GRAM_BF16X3, GRAM_LAG_FP32,
                                              OPT_NEXT_STAGE_MAPS, MAPS_RECOMPUTED, MAPS_STREAMED)
    from paper_2209_13027_amd.workloads import WORKLOADS, make_views

    wl = WORKLOADS[name]
    tg = time.perf_counter()
    v1, v2, cls = make_views(wl)
    gen_s = time.perf_counter() - tg
    M = int(v1.shape[0])
    ctx = Context(0)
    if args.gram != "fp32":
        ctx.set_option(OPT_GRAM_ARITH, GRAM_BF16X3 if args.gram == "bf16x3" else GRAM_LAG_FP32)
    conv_opt = {"auto": CONV_AUTO, "fp32": CONV_FP32, "bf16x3": CONV_BF16X3}[args.conv]
    ctx.set_option(OPT_CONV_ARITH, conv_opt)
    conv_is_split = args.conv == "bf16x3" or (args.conv == "auto" and wl.k >= 5)
    d1, d2, dc = torch.from_numpy(v1).cuda(), torch.from_numpy(v2).cuda(), torch.from_numpy(cls).cuda()
    del v1, v2
    by, bx = wl.blocks
    feat_dtype = {"counts": torch.uint16, "iq_f32": torch.float32, "iq_f16": torch.float16}[args.features]
    feat = torch.empty((M, 2, wl.L1, by, bx, 1 << wl.L2), dtype=feat_dtype, device="cuda")
    batch = wl.extract_batch

    def step():
        model = pipeline.fit(ctx, d1, d2, dc, wl.n_classes, wl.k, wl.L1, wl.L2)
        pipeline.extract(ctx, d1, d2, model["filters"], wl.k, wl.L1, wl.L2, wl.block, wl.stride, batch, out=feat,
                         dtype=feat_dtype, fused=args.fused)

    if args.copy_calibration > 0:
        src = torch.ones(args.copy_calibration * (1 << 18), dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(W):
        step()
    torch.cuda.synchronize()
    ctx.status()

    # timed region: HIP events recorded by the library on its stream around the launches of the dominant kernel
    # (the patch-Gram) only, so that the other launches of a step do not pay for event pairs
    ctx.profile_reset()
    ctx.profile_select(["gram"])
    ctx.profile_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(K):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ctx.profile_enable(False)
    prof_gram = ctx.profile_read()["gram"]

    # a few more steps with every kernel family bracketed by events: the per-kernel figures of `kernels`
    K2 = K if not detail else min(K, 5)
    ctx.profile_reset()
    ctx.profile_select(None)
    ctx.profile_enable(True)
    torch.cuda.synchronize()
    ta = time.perf_counter()
    for _ in range(K2):
        step()
    torch.cuda.synchronize()
    dt_all = time.perf_counter() - ta
    ctx.profile_enable(False)
    prof = ctx.profile_read()
    ctx.status()

    def timed(fn, reps):
        ts = []
        for _ in range(reps):
            torch.cuda.synchronize()
            t = time.perf_counter()
            fn()
            torch.cuda.synchronize()
            ts.append(time.perf_counter() - t)
        return {"ms_mean": sum(ts) / len(ts) * 1e3, "ms_min": min(ts) * 1e3, "reps": reps,
                "images_per_s": M / (sum(ts) / len(ts))}

    phases, dt_plain = {}, None
    plain_path = args.conv == "auto" and args.gram == "fp32" and not args.fused
    if detail:
        # the same region without events, to show their cost
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(K2):
            step()
        torch.cuda.synchronize()
        dt_plain = time.perf_counter() - t1
        # learning and extraction timed apart, one synchronised repetition at a time
        model = pipeline.fit(ctx, d1, d2, dc, wl.n_classes, wl.k, wl.L1, wl.L2)
        phases["learn"] = timed(lambda: pipeline.fit(ctx, d1, d2, dc, wl.n_classes, wl.k, wl.L1, wl.L2), K2)
        phases["extract"] = timed(lambda: pipeline.extract(ctx, d1, d2, model["filters"], wl.k, wl.L1, wl.L2, wl.block,
                                                           wl.stride, batch, out=feat, dtype=feat_dtype,
                                                           fused=args.fused), K2)
        if args.gram != "lag":
            # the same learning with the first stage's maps recomputed inside the second stage's Gram kernel
            # (no maps in memory; the Gram pays for the convolution), for comparison
            ctx.set_option(OPT_NEXT_STAGE_MAPS, MAPS_RECOMPUTED)
            run = lambda: pipeline.fit(ctx, d1, d2, dc, wl.n_classes, wl.k, wl.L1, wl.L2)
            run()
            ctx.profile_reset()
            ctx.profile_select(["gram", "conv"])
            ctx.profile_enable(True)
            phases["learn_maps_recomputed"] = timed(run, K2)
            ctx.profile_enable(False)
            pr = ctx.profile_read()
            phases["learn_maps_recomputed"]["gram_ms"] = pr["gram"]["ms"] / K2
            phases["learn_maps_recomputed"]["conv_ms"] = pr["conv"]["ms"] / K2
            ctx.set_option(OPT_NEXT_STAGE_MAPS, MAPS_STREAMED)
            ctx.profile_reset()
            ctx.profile_enable(True)
            timed(run, K2)
            ctx.profile_enable(False)
            pr = ctx.profile_read()
            phases["learn"]["gram_ms"] = pr["gram"]["ms"] / K2
            phases["learn"]["conv_ms"] = pr["conv"]["ms"] / K2
        if not args.fused:
            # the same extraction with the second stage fused into the output layer, for comparison
            run = lambda: pipeline.extract(ctx, d1, d2, model["filters"], wl.k, wl.L1, wl.L2, wl.block, wl.stride,
                                           batch, out=feat, dtype=feat_dtype, fused=True)
            run()                                             # untimed: first launch loads the kernel
            ctx.profile_reset()
            ctx.profile_select(["conv_hash_hist"])
            ctx.profile_enable(True)
            phases["extract_fused"] = timed(run, K2)
            ctx.profile_enable(False)
            phases["extract_fused"]["conv_hash_hist_ms"] = ctx.profile_read()["conv_hash_hist"]["ms"] / K2
            phases["extract_fused"]["e2e_images_per_s"] = M / ((phases["learn"]["ms_mean"]
                                                                + phases["extract_fused"]["ms_mean"]) * 1e-3)
        if not args.fused:
            # the same extraction with the other convolution arithmetic (same accuracy bars), for comparison
            other, other_name = (CONV_FP32, "fp32") if conv_is_split else (CONV_BF16X3, "bf16x3")
            ctx.set_option(OPT_CONV_ARITH, other)
            run = lambda: pipeline.extract(ctx, d1, d2, model["filters"], wl.k, wl.L1, wl.L2, wl.block, wl.stride,
                                           batch, out=feat, dtype=feat_dtype)
            run()
            ctx.profile_reset()
            ctx.profile_select(["conv"])
            ctx.profile_enable(True)
            phases["extract_conv_other"] = timed(run, K2)
            ctx.profile_enable(False)
            phases["extract_conv_other"]["conv_ms"] = ctx.profile_read()["conv"]["ms"] / K2
            phases["extract_conv_other"]["arithmetic"] = other_name
            ctx.set_option(OPT_CONV_ARITH, conv_opt)
    dense_split = None
    if plain_path:
        # The step as timed above except for the Gram arithmetic: three-piece bf16 operands on the bf16 matrix
        # pipeline (same dense contraction, same parity bars).  Not part of `value`: the path's Gram is the fp32 one.
        ctx.set_option(OPT_GRAM_ARITH, GRAM_BF16X3)
        step()
        ctx.profile_reset()
        ctx.profile_select(["gram"])
        ctx.profile_enable(True)
        reps = min(K2, 5)
        dense_split = timed(step, reps)
        ctx.profile_enable(False)
        g = ctx.profile_read()["gram"]
        dense_split["gram_ms"] = g["ms"] / reps
        work_gram_flops = algorithmic_work(wl, M, feat.element_size())["gram_flops"]
        tf = work_gram_flops / (g["ms"] / reps * 1e-3) / 1e12 if g["ms"] > 0 else 0.0
        dense_split["gram_fp32_equivalent_tflops"] = tf
        dense_split["gram_frac_of_bf16_peak_over_6"] = tf / (PEAK_MFMA_BF16_TFLOPS / 6.0)
        dense_split["options"] = "gram: dense, three-piece bf16 operands (fp32-grade); everything else as in `value`"
        ctx.set_option(OPT_GRAM_ARITH, GRAM_FP32)
    fast = None
    if plain_path:
        # The whole step once more with every widened option on: the lag-structured Gram, three-piece bf16
        # operands in the convolution (same accuracy bars, see the parity tests) and the fused last stage.
        # Not part of `value`.
        ctx.set_option(OPT_CONV_ARITH, CONV_BF16X3)
        ctx.set_option(OPT_GRAM_ARITH, GRAM_LAG_FP32)

        def fast_step():
            mdl = pipeline.fit(ctx, d1, d2, dc, wl.n_classes, wl.k, wl.L1, wl.L2)
            pipeline.extract(ctx, d1, d2, mdl["filters"], wl.k, wl.L1, wl.L2, wl.block, wl.stride, batch, out=feat,
                             dtype=feat_dtype, fused=True)
        fast_step()
        ctx.profile_reset()
        ctx.profile_select(["gram", "conv_hash_hist"])
        ctx.profile_enable(True)
        fast = timed(fast_step, K2)
        ctx.profile_enable(False)
        pf = ctx.profile_read()
        fast["gram_ms"] = pf["gram"]["ms"] / K2
        fast["conv_hash_hist_ms"] = pf["conv_hash_hist"]["ms"] / K2
        fast["options"] = "gram lag-structured fp32, conv bf16x3 (every k), fused last stage (same parity bars)"
        ctx.set_option(OPT_CONV_ARITH, conv_opt)
        ctx.set_option(OPT_GRAM_ARITH, GRAM_FP32)
    ctx.profile_select(None)
    ctx.status()

    work = algorithmic_work(wl, M, feat.element_size())
    L1v, P = wl.L1, wl.h * wl.w
    gram_ms = prof_gram["ms"] / max(1, prof_gram["launches"])
    gram_flops_per_launch = work["gram_flops"] * K / max(1, prof_gram["launches"])
    gram_tflops = gram_flops_per_launch / (gram_ms * 1e-3) / 1e12 if gram_ms > 0 else 0.0
    conv_ms = prof["conv"]["ms"] / K2
    hist_ms = prof["hash_hist"]["ms"] / K2
    fused_ms = prof["conv_hash_hist"]["ms"] / K2
    per = lambda x, ms: x / (ms * 1e-3) if ms > 0 else 0.0
    conv_gbs, conv_tf = per(work["conv_bytes"], conv_ms) / 1e9, per(work["conv_flops"], conv_ms) / 1e12
    kernels = {
        "gram": {"ms_per_step": prof["gram"]["ms"] / K2, "launches_per_step": prof["gram"]["launches"] / K2,
                 "useful_tflops": gram_tflops, "frac_mfma_fp32": gram_tflops / PEAK_MFMA_FP32_TFLOPS},
        "gram_cross": {"ms_per_step": prof["gram_cross"]["ms"] / K2,
                       "launches_per_step": prof["gram_cross"]["launches"] / K2,
                       "useful_tflops": per(work["gram_cross_flops"] * K2, prof["gram_cross"]["ms"]) / 1e12},
        "class_sum": {"ms_per_step": prof["class_sum"]["ms"] / K2,
                      "gbs": per(work["class_sum_bytes"], prof["class_sum"]["ms"] / K2) / 1e9},
        "reduce": {"ms_per_step": prof["reduce"]["ms"] / K2},
        "solve": {"ms_per_step": prof["solve"]["ms"] / K2, "launches_per_step": prof["solve"]["launches"] / K2},
        # the convolution against HBM (algorithmic bytes); its useful fp32-equivalent flop rate beside it (with the
        # fp32 matrix instructions that rate is capped at k/(k+1) of 157.3 TFLOP/s; three-piece bf16 operands run six
        # bf16 instructions per fp32 product set on the 2.5 PFLOP/s pipeline)
        "conv": {"ms_per_step": conv_ms, "gbs": conv_gbs, "frac_hbm": conv_gbs / PEAK_HBM_GBS, "tflops": conv_tf,
                 "arithmetic": "bf16x3" if conv_is_split else "fp32"},
        "hash_hist": {"ms_per_step": hist_ms, "gbs": per(work["hist_bytes"], hist_ms) / 1e9,
                      "frac_hbm": per(work["hist_bytes"], hist_ms) / 1e9 / PEAK_HBM_GBS},
    }
    # measured HBM bytes per launch (committed counter summary) beside the algorithmic ones, for the two memory-bound
    # kernels of the default path: a ratio well above 1 would mean re-reads
    if fused_ms == 0 and prof["conv"]["launches"] > 0 and prof["hash_hist"]["launches"] > 0:
        conv_rx = (r"conv_split_kernel<\d+, \d+, \d+, \d+, (true|false), false>" if conv_is_split
                   else r"conv_mfma_kernel<")
        for key, rx, algo in (("conv", conv_rx, work["conv_bytes"]),
                              ("hash_hist", r"hash_hist_kernel<\d+, \d+, false, (true|false)>", work["hist_bytes"])):
            t = measured_traffic(wl.name, rx)
            kernels[key]["algorithmic_bytes_per_launch"] = algo * K2 / prof[key]["launches"]
            kernels[key]["traffic_bytes_per_launch"] = t
            kernels[key]["traffic_source"] = "profiles/traffic.json (committed, not re-measured)" if t else None
    if "extract_conv_other" in phases:
        # extraction only: stage 1 once per view plus stage 2
        xbytes = 2 * M * P * (4 + 4 * L1v) + 2 * M * L1v * P * (4 + 4 * wl.L2)
        cs = phases["extract_conv_other"]["conv_ms"]
        kernels["conv_%s_extract" % phases["extract_conv_other"]["arithmetic"]] = {
            "ms_per_extract": cs, "gbs": per(xbytes, cs) / 1e9, "frac_hbm": per(xbytes, cs) / 1e9 / PEAK_HBM_GBS}
    if fused_ms > 0:
        # stage-2 conv bytes and flops move from "conv" into the fused kernel
        fused_flops = 2 * M * L1v * P * 2 * wl.D * wl.L2
        fused_bytes = 2 * M * L1v * (P * 4 + by * bx * (1 << wl.L2) * feat.element_size())
        s1_bytes = 2 * (2 * M * P * (4 + 4 * L1v))
        kernels["conv"]["gbs"] = per(s1_bytes, conv_ms) / 1e9
        kernels["conv"]["frac_hbm"] = kernels["conv"]["gbs"] / PEAK_HBM_GBS
        kernels["conv"]["tflops"] = per(2 * (2 * M * P * 2 * wl.D * L1v), conv_ms) / 1e12
        del kernels["hash_hist"]
        kernels["conv_hash_hist"] = {"ms_per_step": fused_ms, "tflops": per(fused_flops, fused_ms) / 1e12,
                                     "frac_mfma_fp32": per(fused_flops, fused_ms) / 1e12 / PEAK_MFMA_FP32_TFLOPS,
                                     "gbs": per(fused_bytes, fused_ms) / 1e9}
    # (the all-tiles, fp32, maps-from-memory instantiation: patch_gram_kernel<k, tsplit, false, waves, false, false, *>, either tile staging)
    traffic = (measured_traffic(wl.name, r"patch_gram_kernel<\d+, \d+, false, \d+, false, false, (true|false)>")
               if args.gram == "fp32" else None)
    # the peak the dominant kernel is held against: the fp32 matrix instructions; with three-piece bf16 operands one
    # fp32 product costs six bf16 products, so the ceiling for fp32-equivalent flop is a sixth of the bf16 peak
    gram_peak, gram_note = PEAK_MFMA_FP32_TFLOPS, None
    if args.gram == "bf16x3":
        gram_peak = PEAK_MFMA_BF16_TFLOPS / 6.0
        gram_note = ("fp32-equivalent flop; peak = dense bf16 matrix peak 2500 TFLOP/s / 6 piece products per fp32 "
                     "product")
    elif args.gram == "lag":
        gram_note = ("flop of the DENSE definition per second: the lag-structured kernel executes (2k-1)^2 lag "
                     "correlations per view pair instead of k^4 products, so this can exceed the peak")
    res = {
        "value": M * K / dt, "ms_per_step": dt / K * 1e3, "steps": K, "warmup": W,
        "config": {"workload": wl.name, "images": M, "classes": wl.n_classes, "h": wl.h, "w": wl.w, "k": wl.k,
                   "L1": wl.L1, "L2": wl.L2, "block": wl.block, "stride": wl.stride, "bins": 1 << wl.L2,
                   "feature_len": wl.feature_len, "features": args.features,
                   "fused_last_stage": bool(args.fused), "conv_arithmetic": "bf16x3 (three-piece, fp32-grade)" if conv_is_split else "fp32",
                   "gram_arithmetic": args.gram, "second_stage_learning": "streamed from the inputs",
                   "input_generation_s": round(gen_s, 1)},
        "roofline": {"bound": "mfma", "kernel": "patch_gram_kernel (all-tiles variant: the Gram over the input maps)",
                     "achieved": gram_tflops, "peak": gram_peak, "unit": "TFLOP/s",
                     "frac": gram_tflops / gram_peak, "traffic": traffic,
                     "traffic_source": ("profiles/traffic.json (rocprofv3 --pmc passes of this command, committed; "
                                        "not re-measured in this run)" if traffic is not None else None),
                     "avg_launch_ms": gram_ms, "launches_per_step": prof_gram["launches"] / K,
                     "algorithmic_flop_per_launch": gram_flops_per_launch},
        "kernels": kernels,
        "kernel_steps": K2,
        "ms_per_step_with_all_kernels_timed": dt_all / K2 * 1e3,
    }
    if gram_note:
        res["roofline"]["note"] = gram_note
    if phases:
        res["phases"] = phases
    if dense_split:
        res["dense_gram_bf16x3_path"] = dense_split
    if fast:
        res["widened_path"] = fast
    if dt_plain is not None:
        res["ms_per_step_without_events"] = dt_plain / K2 * 1e3
    ctx.close()
    del feat, d1, d2, dc
    gc.collect()
    torch.cuda.empty_cache()
    return wl, res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="large_scale", choices=ALL_WORKLOADS,
                    help="the headline workload (value, roofline, cpu_baseline); default: the largest configuration")
    ap.add_argument("--others", default="all",
                    help="'all' (default): also measure the other configurations and report them under "
                         "other_workloads; 'none'; or a comma-separated list of workload names")
    ap.add_argument("--features", default="counts", choices=["counts", "iq_f32", "iq_f16"],
                    help="output layer: uint16 block histograms (the headline path) or the information-quality "
                         "values -log p(t) as fp32 / fp16")
    ap.add_argument("--fused", action="store_true",
                    help="time the path with the second stage convolution fused into the output layer (the "
                         "stage-2 maps are never written); the default materialises them")
    ap.add_argument("--conv", default="auto", choices=["auto", "fp32", "bf16x3"],
                    help="arithmetic of the stage convolution: the library default (three-piece bf16 operands on the "
                         "bf16 matrix pipeline from k = 5 on, fp32 matrix instructions at k = 3; same accuracy), or "
                         "one of the two for every k")
    ap.add_argument("--gram", default="fp32", choices=["fp32", "bf16x3", "lag"],
                    help="arithmetic of the patch-Gram accumulation: fp32 matrix instructions (the headline path), "
                         "three-piece bf16 operands on the bf16 matrix pipeline (same accuracy), or the "
                         "lag-structured form on the fp32 matrix instructions (same accuracy)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-detail", action="store_true", help="skip the comparison legs of the headline workload")
    ap.add_argument("--cpu-images", type=int, default=0, help="images in the CPU-oracle sample (0 = default)")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MIB",
                    help="before the steps, run one plain device copy of this many MiB (a kernel of known "
                         "traffic that scales the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives are part of it); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)

    wl, head = measure(args.workload, args, args.steps, args.warmup, not args.no_detail)
    out = {
        "metric": "images/s for 2-stage DDCCANet extraction (learn both stages + extract features)",
        "value": head.pop("value"), "unit": "images/s", "n_gpus": 1, "steps": head.pop("steps"),
        "warmup": head.pop("warmup"), "ms_per_step": head.pop("ms_per_step"), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
    }
    out.update(head)
    if args.others == "all":
        others = [n for n in ALL_WORKLOADS if n != args.workload]
    elif args.others in ("", "none"):
        others = []
    else:
        others = [n for n in args.others.split(",") if n and n != args.workload]
    if others:
        out["other_workloads"] = {}
        for name in others:
            # steps sized so that a workload's timed region stays within a few seconds
            k_o = max(3, min(args.steps, 20))
            _, res = measure(name, args, k_o, min(args.warmup, 2), False)
            out["other_workloads"][name] = {"images_per_s": res.pop("value"), **res}
    if not args.no_cpu_baseline:
        n_cpu = args.cpu_images or CPU_SAMPLE_IMAGES.get(wl.name, 64)
        out["cpu_baseline"] = run_cpu_baseline(wl, n_cpu)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
