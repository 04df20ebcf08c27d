#!/usr/bin/env python3
"""Benchmark of the masked-convolution hot path on one MI355X.

Workload (config.workload): the ResNet18 stage-1 convolution of the benchmark description --
batch 32, 64->64 channels at 56x56, 3x3 stride 1 pad 1, bf16 with float accumulation, half of
the lowered rows masked out (seeded synthetic tensors, already resident in HBM).

A step is one `sparse_conv_run`: gather of the kept rows, contraction on the matrix cores and
placement into the dense output with zero fill, one fused launch.  The mask -> row-index
compaction belongs to operator setup (the mask is frozen after training) and is timed
separately (`plan_ms`).  `value` = 2*kept*K*Cout / time, the algorithmic TFLOP/s of the kept rows.

Also printed in the same JSON line: the dense run of the same kernels and the speed-up over it
at s in {0.25, 0.5, 0.7}, the roofline of the fused kernel, and the CPU oracle timed on the host
cores (a baseline for scale, not a target).
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

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0

# HBM bytes per launch of the fused kernel on the benchmark workload, from the rocprofv3 --pmc
# runs summarised in profiles/band_alternating_kernel_bf16_resnet18_stage1_s50.md:
# FETCH_SIZE 6890.01 KiB x 1.999 (64 MiB copy calibration) + WRITE_SIZE 12544 KiB x 1.000.
MEASURED_TRAFFIC_BYTES = int(6890.01 * 1024 * 1.999 + 12544 * 1024)


def cpu_baseline(spec, ci, budget_s: float = 12.0):
    """The oracle as it stands, on the host cores, repeated on the benchmark layer until the budget is used."""
    from oracle import oracle

    oracle.masked_conv2d(spec, ci.x, ci.w, ci.bias, ci.mask)  # warm-up (page-in, thread pool)
    reps, t0 = 0, time.perf_counter()
    while True:
        oracle.masked_conv2d(spec, ci.x, ci.w, ci.bias, ci.mask)
        reps += 1
        el = time.perf_counter() - t0
        if el >= budget_s or reps >= 200:
            break
    flops = 2.0 * ci.keep * spec.k * spec.c_out
    return {"value": flops * reps / el / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"whole benchmark layer (kept {ci.keep} of {spec.m} rows), {reps} passes in {el:.1f} s, "
                      "double accumulation"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--with-copy", action="store_true",
                    help="also run a plain 64 MiB device copy 20 times (calibrates HBM counters under rocprofv3)")
    ap.add_argument("--headline-only", action="store_true",
                    help="run only the timed s=0.5 sparse launches (keeps a rocprofv3 kernel summary to one workload)")
    ap.add_argument("--tile", type=str, default="", help="force the sparse tile, e.g. 128x64 (tuning)")
    ap.add_argument("--dense-tile", type=str, default="", help="force the dense tile (tuning)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (the rows of the lowered matrix "
              "are independent, so more GPUs would only split the batch). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch

    import workloads as W
    from paper_2309_06626_amd import binding as B
    from paper_2309_06626_amd import runtime as R
    from paper_2309_06626_amd.metrics import algorithmic_bytes, buffer_sets_for_cold_runs, time_launches, time_rotating

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    B.lib()

    results = {}
    headline = None
    sparsities = (0.5,) if args.headline_only else (0.5, 0.25, 0.7)
    for s in sparsities:
        spec = W.config2(s)
        ci = W.make_conv_inputs(spec, W.base_seed(2))
        t0 = time.perf_counter()
        layer = R.ConvLayer(spec, ci.w, ci.bias, ci.mask)
        torch.cuda.synchronize()
        plan_ms = (time.perf_counter() - t0) * 1e3
        if args.tile:
            B.sparse_conv_plan_set_tiles(layer.plan, 0, *map(int, args.tile.split("x")))
        if args.dense_tile:
            B.sparse_conv_plan_set_tiles(layer.plan, 1, *map(int, args.dense_tile.split("x")))
        x = R.to_device(ci.x, spec.dtype)
        y = layer.new_output()
        steps = args.steps if s == 0.5 else max(args.steps // 4, 50)
        warm = args.warmup if s == 0.5 else max(args.warmup // 4, 10)
        wall_s, ev_s = time_launches(B.prepared_run(layer.plan, x, layer.bias, y), steps, warm)
        if args.headline_only:
            wall_d, ev_d = float("nan"), float("nan")
        else:
            wall_d, ev_d = time_launches(B.prepared_run(layer.plan, x, layer.bias, y, dense=True),
                                         max(steps // 4, 50), max(warm // 4, 10))
        cold = None
        if s == 0.5 and not args.headline_only:
            # cold regime: the launches rotate through copies of x and y totalling 768 MB, so nothing is
            # served from the 256 MB memory-side cache (the warm figures above keep one 26 MB working set)
            nsets = buffer_sets_for_cold_runs(x.numel() * x.element_size() + y.numel() * y.element_size())
            xs = [x] + [x.clone() for _ in range(nsets - 1)]
            ys = [y] + [torch.empty_like(y) for _ in range(nsets - 1)]
            ev_c = time_rotating([B.prepared_run(layer.plan, a, layer.bias, b) for a, b in zip(xs, ys)],
                                 max(steps // 4, 2 * nsets), nsets)
            ev_cd = time_rotating([B.prepared_run(layer.plan, a, layer.bias, b, dense=True) for a, b in zip(xs, ys)],
                                  max(steps // 4, 2 * nsets), nsets)
            cold = {"kernel_us": ev_c * 1e6, "dense_kernel_us": ev_cd * 1e6, "speedup_vs_dense": ev_cd / ev_c,
                    "buffer_sets": nsets}
            del xs, ys
        results[s] = dict(spec=spec, ci=ci, layer=layer, wall=wall_s, ev=ev_s, wall_dense=wall_d, ev_dense=ev_d,
                          plan_ms=plan_ms, steps=steps, warm=warm, cold=cold)
        if s == 0.5:
            headline = results[s]

    if args.with_copy:
        src = torch.empty(64 << 20, dtype=torch.uint8, device="cuda:0").zero_()
        dst = torch.empty_like(src)
        for _ in range(20):
            dst.copy_(src)
        torch.cuda.synchronize()

    r = headline
    spec, ci = r["spec"], r["ci"]
    flops = 2.0 * ci.keep * spec.k * spec.c_out
    flops_dense = 2.0 * spec.m * spec.k * spec.c_out
    value = flops / r["wall"] / 1e12
    abytes = algorithmic_bytes(spec, ci.keep)
    achieved = abytes / r["ev"] / 1e9
    tm, tn, wgs = B.sparse_conv_plan_tiles(r["layer"].plan, 0)
    dm, dn, dwgs = B.sparse_conv_plan_tiles(r["layer"].plan, 1)
    kernel = B.sparse_conv_plan_kernel(r["layer"].plan, 0)
    out = {
        "metric": "sparse-conv TFLOP/s (algorithmic, kept rows) at s=0.5; speed-up vs dense at s in {0.25,0.5,0.7}",
        "value": value,
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": r["steps"],
        "warmup": r["warm"],
        "ms_per_step": r["wall"] * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "configs[1]: ResNet18 stage-1 conv, batch 32, 64->64 @56x56, 3x3 s1 p1, bf16, "
                               "row mask s=0.5 (kept 50176 of 100352 rows), NHWC, bias+ReLU, zero fill",
                   "m": spec.m, "k": spec.k, "c_out": spec.c_out, "kept": ci.keep,
                   "kernel_sparse": kernel, "kernel_dense": B.sparse_conv_plan_kernel(r["layer"].plan, 1),
                   "tile_sparse": f"{tm}x{tn}", "workgroups_sparse": wgs,
                   "tile_dense": f"{dm}x{dn}", "workgroups_dense": dwgs},
        "kernel_us": r["ev"] * 1e6,
        "dense_kernel_us": r["ev_dense"] * 1e6,
        "dense_tflops": flops_dense / r["wall_dense"] / 1e12,
        "speedup_vs_dense": {str(s): results[s]["ev_dense"] / results[s]["ev"] for s in sorted(results)},
        "sparse_tflops_by_s": {str(s): 2.0 * results[s]["ci"].keep * spec.k * spec.c_out / results[s]["wall"] / 1e12
                               for s in sorted(results)},
        "mfma_peak_frac": flops / r["ev"] / 1e12 / MFMA_BF16_PEAK_TFLOPS,
        "plan_ms": r["plan_ms"],
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": MEASURED_TRAFFIC_BYTES,
                     "algorithmic_bytes": abytes,
                     "kernel": f"{kernel} (one fused launch: lowering of the kept windows inside LDS, MFMA, scatter, zero fill)"},
    }
    if r["cold"]:
        c = dict(r["cold"])
        c["tflops"] = flops / (c["kernel_us"] * 1e-6) / 1e12
        c["achieved_gbs"] = abytes / (c["kernel_us"] * 1e-6) / 1e9
        c["hbm_frac"] = c["achieved_gbs"] / HBM_PEAK_GBS
        out["cold_cache"] = c
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(spec, ci)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
