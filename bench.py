#!/usr/bin/env python3
"""Benchmark of the masked-convolution hot path on one MI355X.

Workload (config.workload): the ResNet18 stage-1 convolution of the benchmark description --
batch 32, 64->64 channels at 56x56, 3x3 stride 1 pad 1, bf16 with float accumulation, half of
the lowered rows masked out (seeded synthetic tensors, already resident in HBM).

A step is one `sparse_conv_run`: gather of the kept rows, contraction on the matrix cores and
placement into the dense output with zero fill, one fused launch.  The mask -> row-index
compaction belongs to operator setup (the mask is frozen after training) and is timed
separately (`plan_ms`).  `value` = 2*kept*K*Cout / time, the algorithmic TFLOP/s of the kept rows.

Timing: the K steps are recorded once as a HIP graph of K launches (the launch-bound inner loop
of a serving process) and replayed; a repeat is W untimed warm-up steps and one replay of the K
steps bracketed by device synchronisations; `ms_per_step` is the median over the repeats (wall
clock), `kernel_us` the median of the same replays' event times on the launch stream.

Also printed in the same JSON line: the dense run of the same kernels and the speed-up over it
at s in {0.25, 0.5, 0.7}, the roofline of the fused kernel beside the measured ceilings of the
device (plain copy, register-resident MFMA loop), the cold-cache regime, and the CPU oracle timed
on the host cores (a baseline for scale, not a target).
"""
from __future__ import annotations

import argparse
import json
import os
import re
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
REPEATS = 7

# rocprofv3 summary of this benchmark's dominant kernel: bench.py reads the HBM bytes per launch that the
# FETCH_SIZE / WRITE_SIZE counter runs measured from it (the line "traffic_bytes_per_launch: N"), together
# with the kernel it was measured for; a kernel that no longer matches yields traffic = null.
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "band_tap_kernel_bf16_resnet18_stage1_s50.md")


def measured_traffic(kernel: str):
    try:
        text = open(TRAFFIC_PROFILE).read()
    except OSError:
        return None, None
    m = re.search(r"traffic_bytes_per_launch:\s*(\d+)", text)
    k = re.search(r"traffic_measured_for_kernel:\s*(\S+)", text)
    if not m or not k or k.group(1) != kernel:
        return None, None
    return int(m.group(1)), os.path.relpath(TRAFFIC_PROFILE, ROOT)


def cpu_baseline(spec, ci, budget_s: float = 12.0):
    """The oracle as it stands, on the host cores, repeated on the benchmark layer until the budget is used;
    then one pass on a single thread."""
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
    out = {"value": flops * reps / el / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
           "sample": f"whole benchmark layer (kept {ci.keep} of {spec.m} rows), {reps} passes in {el:.1f} s, "
                     "double accumulation"}
    # the same oracle on one thread (a child process: the OpenMP thread count is fixed when the library loads)
    import subprocess

    code = ("import time, workloads as W\nfrom oracle import oracle\nspec = W.config2(0.5)\n"
            "ci = W.make_conv_inputs(spec, W.base_seed(2))\noracle.masked_conv2d(spec, ci.x, ci.w, ci.bias, ci.mask)\n"
            "t0 = time.perf_counter()\noracle.masked_conv2d(spec, ci.x, ci.w, ci.bias, ci.mask)\n"
            "print('SINGLE', time.perf_counter() - t0, oracle.num_threads())\n")
    try:
        r = subprocess.run([sys.executable, "-c", code], cwd=ROOT, env=dict(os.environ, OMP_NUM_THREADS="1"),
                           capture_output=True, text=True, timeout=120)
        for line in r.stdout.splitlines():
            if line.startswith("SINGLE"):
                _, sec, thr = line.split()
                if int(thr) == 1:
                    out["single_thread_tflops"] = flops / float(sec) / 1e12
    except (subprocess.SubprocessError, OSError, ValueError):
        pass
    return out


def median_times(call, steps: int, warmup: int, repeats: int = REPEATS):
    from paper_2309_06626_amd.metrics import LaunchGraph

    g = LaunchGraph(call, steps)
    runs = [g.replay(warmup) for _ in range(repeats)]
    wall = statistics.median(r[0] for r in runs) / steps
    ev = statistics.median(r[1] for r in runs) / steps
    return wall, ev, [r[1] / steps for r in runs]


def device_ceilings():
    """Measured ceilings of this device: HBM read + write GB/s of a plain copy (1 GiB moved per launch: beyond the
    256 MB memory-side cache) and TFLOP/s of a register-resident bf16 MFMA loop on every compute unit."""
    import torch

    from paper_2309_06626_amd import binding as B

    n = 512 << 20
    src = torch.empty(n, dtype=torch.uint8, device="cuda:0").fill_(1)
    dst = torch.empty_like(src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(3):
        B.sc_probe_stream_copy(dst, src)
    best_copy = 0.0
    for _ in range(5):
        e0.record()
        for _ in range(4):
            B.sc_probe_stream_copy(dst, src)
        e1.record()
        torch.cuda.synchronize()
        best_copy = max(best_copy, 4 * 2.0 * n / (e0.elapsed_time(e1) * 1e-3) / 1e9)
    del src, dst
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    wgs = cus * 4                                  # four workgroups of four wavefronts: four wavefronts per SIMD
    out = torch.empty(wgs * 256, dtype=torch.float32, device="cuda:0")
    B.sc_probe_mfma_bf16(2000, wgs, out)
    best_mfma = 0.0
    for _ in range(5):
        e0.record()
        flops = B.sc_probe_mfma_bf16(20000, wgs, out)
        e1.record()
        torch.cuda.synchronize()
        best_mfma = max(best_mfma, flops / (e0.elapsed_time(e1) * 1e-3) / 1e12)
    return {"hbm_copy_gbs": best_copy, "mfma_bf16_tflops": best_mfma, "compute_units": cus,
            "how": "plain 16-byte copy of 512 MiB (read + write counted); 32x32x16 bf16 MFMA loop on register operands, "
                   "16 wavefronts per compute unit; best of 5"}


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
    ap.add_argument("--eager", action="store_true", help="launch step by step from the host instead of replaying a graph "
                    "(profiling runs: every launch is a separate dispatch either way, but counters attach per launch)")
    ap.add_argument("--no-tune", action="store_true", help="keep the cost model's kernel choice (no measured choice)")
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
    from paper_2309_06626_amd.metrics import algorithmic_bytes, buffer_sets_for_cold_runs, time_rotating

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    B.lib()

    def eager_times(fn, steps, warmup):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        for _ in range(steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps, e0.elapsed_time(e1) * 1e-3 / steps

    def timed(call, steps, warm):
        if args.eager:
            w, e = eager_times(call, steps, warm)
            return w, e, [e]
        return median_times(call, steps, warm)

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
        tune_ms = None
        if not args.no_tune:
            t0 = time.perf_counter()
            B.sparse_conv_plan_tune(layer.plan, x, layer.bias, y)
            tune_ms = (time.perf_counter() - t0) * 1e3
        call_s = B.prepared_run(layer.plan, x, layer.bias, y)
        call_d = B.prepared_run(layer.plan, x, layer.bias, y, dense=True)
        # clocks: a quarter of a second of launches before anything is timed (short runs otherwise measure the ramp)
        t_end = time.perf_counter() + 0.25
        while time.perf_counter() < t_end:
            for _ in range(200):
                call_s()
            torch.cuda.synchronize()
        steps = args.steps if s == 0.5 else max(args.steps // 4, 50)
        warm = args.warmup if s == 0.5 else max(args.warmup // 4, 10)
        wall_s, ev_s, reps_s = timed(call_s, steps, warm)
        if args.headline_only:
            wall_d, ev_d = float("nan"), float("nan")
        else:
            wall_d, ev_d, _ = timed(call_d, max(steps // 4, 50), max(warm // 4, 10))
        cold = None
        if s == 0.5 and not args.headline_only:
            # cold regime: the launches rotate through copies of x and y totalling 768 MB, so nothing is
            # served from the 256 MB memory-side cache (the warm figures above keep one 26 MB working set)
            nsets = buffer_sets_for_cold_runs(x.numel() * x.element_size() + y.numel() * y.element_size())
            xs = [x] + [x.clone() for _ in range(nsets - 1)]
            ys = [y] + [torch.empty_like(y) for _ in range(nsets - 1)]
            cs = [B.prepared_run(layer.plan, a, layer.bias, b) for a, b in zip(xs, ys)]
            cd = [B.prepared_run(layer.plan, a, layer.bias, b, dense=True) for a, b in zip(xs, ys)]
            n_cold = max(steps // 4, 4 * nsets)
            ev_c = time_rotating(cs, n_cold, nsets, repeats=5)
            ev_cd = time_rotating(cd, n_cold, nsets, repeats=5)
            cold = {"kernel_us": ev_c * 1e6, "dense_kernel_us": ev_cd * 1e6, "speedup_vs_dense": ev_cd / ev_c,
                    "buffer_sets": nsets, "how": "graph of launches rotating through the buffer sets, median of 5 replays"}
            del xs, ys, cs, cd
        results[s] = dict(spec=spec, ci=ci, layer=layer, wall=wall_s, ev=ev_s, wall_dense=wall_d, ev_dense=ev_d,
                          plan_ms=plan_ms, tune_ms=tune_ms, steps=steps, warm=warm, cold=cold, reps=reps_s)
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
    traffic, traffic_source = measured_traffic(kernel)
    ceilings = None if args.headline_only else device_ceilings()
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
                   "tile_dense": f"{dm}x{dn}", "workgroups_dense": dwgs,
                   "launch": "eager" if args.eager else f"HIP graph of {r['steps']} launches, median of {REPEATS} replays",
                   "kernel_choice": "cost model" if args.no_tune else "measured (sparse_conv_plan_tune)"},
        "kernel_us": r["ev"] * 1e6,
        "kernel_us_repeats": [t * 1e6 for t in r["reps"]],
        "dense_kernel_us": r["ev_dense"] * 1e6,
        "dense_tflops": flops_dense / r["wall_dense"] / 1e12,
        "speedup_vs_dense": {str(s): results[s]["ev_dense"] / results[s]["ev"] for s in sorted(results)},
        "sparse_tflops_by_s": {str(s): 2.0 * results[s]["ci"].keep * spec.k * spec.c_out / results[s]["wall"] / 1e12
                               for s in sorted(results)},
        "mfma_peak_frac": flops / r["ev"] / 1e12 / MFMA_BF16_PEAK_TFLOPS,
        "plan_ms": r["plan_ms"],
        "tune_ms": r["tune_ms"],
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_source,
                     "algorithmic_bytes": abytes,
                     "kernel": f"{kernel} (one fused launch: lowering of the kept windows inside LDS, MFMA, scatter, zero fill)"},
    }
    if ceilings:
        out["measured_ceilings"] = ceilings
        out["roofline"]["frac_of_measured_copy"] = achieved / ceilings["hbm_copy_gbs"]
        out["mfma_frac_of_measured_loop"] = flops / r["ev"] / 1e12 / ceilings["mfma_bf16_tflops"]
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
