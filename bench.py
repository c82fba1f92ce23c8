#!/usr/bin/env python3
"""Benchmark of the two-stage DDCCANet hot path on one MI355X.

One "step" = the whole path on one synthetic workload, inputs already in HBM:
  learn stage-1 filters -> apply stage 1 (both views) -> learn stage-2 filters on the maps
  -> extract_features (stage-1 conv, stage-2 conv, hashing + block histograms) for all images.
Prints ONE JSON line: images/s, the roofline of the dominant kernel (patch-Gram, fp32 MFMA),
per-kernel figures, and the CPU oracle timed on a bounded sample of the same workload.
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

PEAK_MFMA_FP32_TFLOPS = 157.3      # MI355X dense fp32 matrix peak
PEAK_HBM_GBS = 8000.0              # MI355X HBM3E
PEAK_FP32_VALU_TFLOPS = 157.3


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


def measured_traffic(workload, kernel_prefix, must_contain=""):
    """HBM bytes per launch (read + write) of the kernels whose name starts with `kernel_prefix`, from the
    rocprofv3 --pmc passes summarised in profiles/traffic.json (FETCH_SIZE / WRITE_SIZE scaled by a plain
    copy of known size); None when no profile of this workload is committed."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    if not os.path.exists(path):
        return None
    with open(path) as f:
        data = json.load(f).get(workload)
    if not data:
        return None
    tot_bytes, tot_launches = 0.0, 0
    for name, v in data.items():
        if name.startswith(kernel_prefix) and must_contain in name and "read_mib_per_launch" in v:
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
        "sample": f"{n} of {wl.M} images ({per_class} per class), whole path (learn both stages + extract), "
                  f"fp64, {dt:.1f} s",
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="small_face")
    ap.add_argument("--features", default="counts", choices=["counts", "iq_f32", "iq_f16"],
                    help="output layer: uint16 block histograms (the headline path) or the information-quality "
                         "values -log p(t) as fp32 / fp16")
    ap.add_argument("--fused", action="store_true",
                    help="time the path with the second stage convolution fused into the output layer (the "
                         "stage-2 maps are never written); the default materialises them")
    ap.add_argument("--conv", default="fp32", choices=["fp32", "bf16x3"],
                    help="arithmetic of the stage convolution: fp32 matrix instructions (the headline path) or "
                         "three-piece bf16 operands on the bf16 matrix pipeline (same accuracy)")
    ap.add_argument("--gram", default="fp32", choices=["fp32", "bf16x3", "lag"],
                    help="arithmetic of the patch-Gram accumulation: fp32 matrix instructions (the headline path), "
                         "three-piece bf16 operands on the bf16 matrix pipeline (same accuracy), or the "
                         "lag-structured form on the fp32 matrix instructions (same accuracy)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
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
    from paper_2209_13027_amd import pipeline
    from paper_2209_13027_amd.binding import Context
    from paper_2209_13027_amd.workloads import WORKLOADS, make_views

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    wl = WORKLOADS[args.workload]
    v1, v2, cls = make_views(wl)
    M = int(v1.shape[0])
    ctx = Context(0)
    if args.gram != "fp32":
        from paper_2209_13027_amd.binding import OPT_GRAM_ARITH, GRAM_BF16X3, GRAM_LAG_FP32
        ctx.set_option(OPT_GRAM_ARITH, GRAM_BF16X3 if args.gram == "bf16x3" else GRAM_LAG_FP32)
    if args.conv == "bf16x3":
        from paper_2209_13027_amd.binding import OPT_CONV_ARITH, CONV_BF16X3
        ctx.set_option(OPT_CONV_ARITH, CONV_BF16X3)
    d1, d2, dc = torch.from_numpy(v1).cuda(), torch.from_numpy(v2).cuda(), torch.from_numpy(cls).cuda()
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
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ctx.status()

    # timed region: HIP events recorded by the library on its stream around the launches of the dominant kernel
    # (the patch-Gram) only, so that the other sixty launches of a step do not pay for event pairs
    ctx.profile_reset()
    ctx.profile_select(["gram"])
    ctx.profile_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ctx.profile_enable(False)
    prof_gram = ctx.profile_read()["gram"]

    # the same steps with every kernel family bracketed by events: the per-kernel figures of `kernels`
    ctx.profile_reset()
    ctx.profile_select(None)
    ctx.profile_enable(True)
    torch.cuda.synchronize()
    ta = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt_all = time.perf_counter() - ta
    ctx.profile_enable(False)
    prof = ctx.profile_read()

    # the same region once more without events, to show their cost
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt_plain = time.perf_counter() - t1
    ctx.status()

    # learning and extraction timed apart, one synchronised repetition at a time (mean and min over K)
    def timed(fn):
        ts = []
        for _ in range(args.steps):
            torch.cuda.synchronize()
            t = time.perf_counter()
            fn()
            torch.cuda.synchronize()
            ts.append(time.perf_counter() - t)
        return {"ms_mean": sum(ts) / len(ts) * 1e3, "ms_min": min(ts) * 1e3,
                "images_per_s": M / (sum(ts) / len(ts))}
    model = pipeline.fit(ctx, d1, d2, dc, wl.n_classes, wl.k, wl.L1, wl.L2)
    phases = {
        "learn": timed(lambda: pipeline.fit(ctx, d1, d2, dc, wl.n_classes, wl.k, wl.L1, wl.L2)),
        "extract": timed(lambda: pipeline.extract(ctx, d1, d2, model["filters"], wl.k, wl.L1, wl.L2, wl.block,
                                                  wl.stride, batch, out=feat, dtype=feat_dtype,
                                                  fused=args.fused)),
        "e2e": timed(step),
    }
    # the same step captured once into a HIP graph and replayed (same kernels, no launch gaps)
    from paper_2209_13027_amd.binding import (OPT_CONV_ARITH as _OC, CONV_BF16X3 as _CB, OPT_GRAM_ARITH as _OG,
                                              GRAM_BF16X3 as _GB, GRAM_LAG_FP32 as _GL)
    opts = ([(_OC, _CB)] if args.conv == "bf16x3" else []) + ([(_OG, _GB)] if args.gram == "bf16x3" else []) + \
           ([(_OG, _GL)] if args.gram == "lag" else [])
    graphed = pipeline.GraphedPath(d1, d2, dc, wl.n_classes, wl.k, wl.L1, wl.L2, wl.block, wl.stride,
                                   batch_images=batch, dtype=feat_dtype, fused=args.fused, out=feat, options=opts)
    graphed.replay()
    graphed.status()
    phases["e2e_graph"] = timed(graphed.replay)
    torch.cuda.synchronize()
    tg = time.perf_counter()
    for _ in range(args.steps):
        graphed.replay()
    torch.cuda.synchronize()
    phases["e2e_graph"]["ms_back_to_back"] = (time.perf_counter() - tg) / args.steps * 1e3
    graphed.status()
    graphed.close()
    del graphed
    if not args.fused:
        # the same extraction with the second stage fused into the output layer, for comparison
        pipeline.extract(ctx, d1, d2, model["filters"], wl.k, wl.L1, wl.L2, wl.block, wl.stride, batch, out=feat,
                         dtype=feat_dtype, fused=True)          # untimed: first launch loads the kernel
        ctx.profile_reset()
        ctx.profile_select(["conv_hash_hist"])
        ctx.profile_enable(True)
        phases["extract_fused"] = timed(lambda: pipeline.extract(ctx, d1, d2, model["filters"], wl.k, wl.L1, wl.L2,
                                                                 wl.block, wl.stride, batch, out=feat,
                                                                 dtype=feat_dtype, fused=True))
        ctx.profile_enable(False)
        pf = ctx.profile_read()["conv_hash_hist"]
        phases["extract_fused"]["conv_hash_hist_ms"] = pf["ms"] / args.steps
        phases["extract_fused"]["e2e_images_per_s"] = M / ((phases["learn"]["ms_mean"]
                                                            + phases["extract_fused"]["ms_mean"]) * 1e-3)
    conv_split = None
    if args.conv == "fp32" and not args.fused:
        # the same extraction with the three-piece bf16 convolution (same accuracy), for comparison
        from paper_2209_13027_amd.binding import OPT_CONV_ARITH, CONV_BF16X3, CONV_FP32
        ctx.set_option(OPT_CONV_ARITH, CONV_BF16X3)
        run = lambda: pipeline.extract(ctx, d1, d2, model["filters"], wl.k, wl.L1, wl.L2, wl.block, wl.stride,
                                       batch, out=feat, dtype=feat_dtype)
        run()
        ctx.profile_reset()
        ctx.profile_select(["conv"])
        ctx.profile_enable(True)
        phases["extract_conv_bf16x3"] = timed(run)
        ctx.profile_enable(False)
        conv_split = ctx.profile_read()["conv"]["ms"] / args.steps
        ctx.set_option(OPT_CONV_ARITH, CONV_FP32)
    fast = None
    if args.conv == "fp32" and args.gram == "fp32" and not args.fused:
        # The whole step once more with every widened option on: the lag-structured Gram, three-piece bf16
        # operands in the convolution (same accuracy bars, see the parity tests) and the fused last stage.
        # Not part of `value`.
        from paper_2209_13027_amd.binding import (OPT_CONV_ARITH, CONV_BF16X3, CONV_FP32, OPT_GRAM_ARITH,
                                                  GRAM_FP32, GRAM_LAG_FP32)
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
        fast = timed(fast_step)
        ctx.profile_enable(False)
        pf = ctx.profile_read()
        fast["gram_ms"] = pf["gram"]["ms"] / args.steps
        fast["gram_useful_tflops"] = (algorithmic_work(wl, M)["gram_flops"] / (fast["gram_ms"] * 1e-3) / 1e12
                                      if fast["gram_ms"] > 0 else 0.0)
        fast["gram_useful_tflops_note"] = ("flop of the dense formulation per second of Gram time: above the fp32 "
                                           "MFMA peak when the lag-structured form does the work")
        fast["conv_hash_hist_ms"] = pf["conv_hash_hist"]["ms"] / args.steps
        fast["options"] = "gram lag-structured fp32, conv bf16x3, fused last stage"
        ctx.set_option(OPT_CONV_ARITH, CONV_FP32)
        ctx.set_option(OPT_GRAM_ARITH, GRAM_FP32)
    ctx.profile_select(None)
    ctx.status()

    work = algorithmic_work(wl, M, feat.element_size())
    L1v, P = wl.L1, wl.h * wl.w
    K = args.steps
    gram_ms = prof_gram["ms"] / max(1, prof_gram["launches"])
    gram_flops_per_launch = work["gram_flops"] * K / max(1, prof_gram["launches"])
    gram_tflops = gram_flops_per_launch / (gram_ms * 1e-3) / 1e12 if gram_ms > 0 else 0.0
    conv_ms = prof["conv"]["ms"] / K
    hist_ms = prof["hash_hist"]["ms"] / K
    fused_ms = prof["conv_hash_hist"]["ms"] / K
    fused_flops = 2 * M * L1v * P * 2 * wl.D * wl.L2
    fused_bytes = 2 * M * L1v * (P * 4 + by * bx * (1 << wl.L2) * feat.element_size())
    kernels = {
        "gram": {"ms_per_step": prof["gram"]["ms"] / K, "launches_per_step": prof["gram"]["launches"] / K,
                 "useful_tflops": gram_tflops, "frac_mfma_fp32": gram_tflops / PEAK_MFMA_FP32_TFLOPS},
        "gram_cross": {"ms_per_step": prof["gram_cross"]["ms"] / K,
                       "launches_per_step": prof["gram_cross"]["launches"] / K,
                       "useful_tflops": work["gram_cross_flops"] * K / (prof["gram_cross"]["ms"] * 1e-3) / 1e12
                       if prof["gram_cross"]["ms"] > 0 else 0.0},
        "class_sum": {"ms_per_step": prof["class_sum"]["ms"] / K,
                      "gbs": work["class_sum_bytes"] / (prof["class_sum"]["ms"] / K * 1e-3) / 1e9
                      if prof["class_sum"]["ms"] > 0 else 0.0},
        "reduce": {"ms_per_step": prof["reduce"]["ms"] / K},
        "solve": {"ms_per_step": prof["solve"]["ms"] / K, "launches_per_step": prof["solve"]["launches"] / K},
        "conv": {"ms_per_step": conv_ms, "gbs": work["conv_bytes"] / (conv_ms * 1e-3) / 1e9 if conv_ms > 0 else 0.0,
                 "frac_hbm": work["conv_bytes"] / (conv_ms * 1e-3) / 1e9 / PEAK_HBM_GBS if conv_ms > 0 else 0.0,
                 "tflops": work["conv_flops"] / (conv_ms * 1e-3) / 1e12 if conv_ms > 0 else 0.0},
        "hash_hist": {"ms_per_step": hist_ms,
                      "gbs": work["hist_bytes"] / (hist_ms * 1e-3) / 1e9 if hist_ms > 0 else 0.0,
                      "frac_hbm": work["hist_bytes"] / (hist_ms * 1e-3) / 1e9 / PEAK_HBM_GBS if hist_ms > 0 else 0.0},
    }
    if conv_split:
        # extraction only: stage 1 once per view plus stage 2
        xbytes = 2 * M * P * (4 + 4 * L1v) + 2 * M * L1v * P * (4 + 4 * wl.L2)
        kernels["conv_bf16x3_extract"] = {"ms_per_extract": conv_split, "gbs": xbytes / (conv_split * 1e-3) / 1e9,
                                          "frac_hbm": xbytes / (conv_split * 1e-3) / 1e9 / PEAK_HBM_GBS}
    if fused_ms > 0:
        # stage-2 conv bytes and flops move from "conv" into the fused kernel
        s1_bytes = 2 * (2 * M * P * (4 + 4 * L1v))
        kernels["conv"]["gbs"] = s1_bytes / (conv_ms * 1e-3) / 1e9 if conv_ms > 0 else 0.0
        kernels["conv"]["frac_hbm"] = kernels["conv"]["gbs"] / PEAK_HBM_GBS
        kernels["conv"]["tflops"] = 2 * (2 * M * P * 2 * wl.D * L1v) / (conv_ms * 1e-3) / 1e12 if conv_ms > 0 else 0.0
        del kernels["hash_hist"]
        kernels["conv_hash_hist"] = {"ms_per_step": fused_ms, "tflops": fused_flops / (fused_ms * 1e-3) / 1e12,
                                     "frac_mfma_fp32": fused_flops / (fused_ms * 1e-3) / 1e12 / PEAK_MFMA_FP32_TFLOPS,
                                     "gbs": fused_bytes / (fused_ms * 1e-3) / 1e9}
    out = {
        "metric": "images/s for 2-stage DDCCANet extraction (learn both stages + extract features)",
        "value": M * K / dt, "unit": "images/s", "n_gpus": 1, "steps": K, "warmup": args.warmup,
        "ms_per_step": dt / K * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": wl.name, "images": M, "classes": wl.n_classes, "h": wl.h, "w": wl.w, "k": wl.k,
                   "L1": wl.L1, "L2": wl.L2, "block": wl.block, "stride": wl.stride, "bins": 1 << wl.L2,
                   "feature_len": wl.feature_len, "features": args.features,
                   "fused_last_stage": bool(args.fused), "conv_arithmetic": args.conv,
                   "gram_arithmetic": args.gram},
        "roofline": {"bound": "mfma", "kernel": "patch_gram_kernel (all-tiles variant: the Gram over the input maps)", "achieved": gram_tflops,
                     "peak": PEAK_MFMA_FP32_TFLOPS, "unit": "TFLOP/s", "frac": gram_tflops / PEAK_MFMA_FP32_TFLOPS,
                     "traffic": measured_traffic(wl.name, "patch_gram_kernel", ", false,"), "avg_launch_ms": gram_ms,
                     "algorithmic_flop_per_launch": gram_flops_per_launch},
        "kernels": kernels,
        "phases": phases,
        "widened_path": fast,
        "ms_per_step_without_events": dt_plain / K * 1e3,
        "ms_per_step_with_all_kernels_timed": dt_all / K * 1e3,
    }
    if not args.no_cpu_baseline:
        default_images = {"tiny": 40, "small_face": 400, "object": 128, "large_scale": 257, "stress": 16}
        n_cpu = args.cpu_images or default_images.get(wl.name, 64)
        out["cpu_baseline"] = run_cpu_baseline(wl, n_cpu)
    ctx.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
