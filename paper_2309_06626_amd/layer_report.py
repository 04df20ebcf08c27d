#!/usr/bin/env python3
"""Per-layer report over the five benchmark configurations on one MI355X.

    python -m paper_2309_06626_amd.layer_report [--configs 1,2,3,4,5] [--steps 200] [--json out.jsonl] [--library-conv]

For every convolution: kernel chosen for the sparse and the dense run, time per launch, algorithmic
TFLOP/s of the kept rows (2*kept*K*Cout / t) and its share of the MFMA peak, algorithmic GB/s and
its share of the HBM peak, and the speed-up over the dense run of the same kernels.  Config 2 is
reported at s in {0, 0.25, 0.5, 0.7} in zero-fill mode and, for s > 0, in scatter-only mode.
Configs 3 and 5 add the time of the whole chain (conv launches plus the pooling / residual glue),
launched call by call and replayed as a HIP graph.
Layers are timed one by one on synthetic inputs of their own shape, back-to-back launches on one
stream, in two cache regimes: warm (the same buffers every launch: working sets of tens of MB stay
in the 256 MB memory-side cache, as they do between the layers of a network) and cold (the launches
rotate through copies of the activations and outputs totalling 768 MB, so operands come from HBM).
"""
from __future__ import annotations

import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


TUNE = True      # measured kernel choice before the timings (main() clears it for --no-tune)


def kernel_name(plan, which):
    from paper_2309_06626_amd import binding as B

    tm, tn, wgs = B.sparse_conv_plan_tiles(plan, which)
    shape = f"{-tm} rows x {tn} ch" if tm < 0 else f"{tm}x{tn}"
    return f"{B.sparse_conv_plan_kernel(plan, which)} {shape} ({wgs} wg)"


def library_conv_us(spec, steps):
    """Context only: torch.nn.functional.conv2d (MIOpen) on the same shape, channels-last, bias included,
    no activation -- shows that the dense run the speed-ups are quoted against is not a weak baseline."""
    import torch
    import torch.nn.functional as F

    from paper_2309_06626_amd import binding as B

    torch.backends.cudnn.benchmark = True    # let the library search its algorithms: the fairest context figure
    dt = B.TORCH_DTYPE[spec.dtype]
    x = torch.randn(spec.n, spec.c_in, spec.h, spec.w, device="cuda:0", dtype=dt).relu_().contiguous(
        memory_format=torch.channels_last)
    w = torch.randn(spec.c_out, spec.c_in, spec.kh, spec.kw, device="cuda:0", dtype=dt).contiguous(
        memory_format=torch.channels_last)
    b = torch.randn(spec.c_out, device="cuda:0", dtype=dt)

    def run():
        return F.conv2d(x, w, b, stride=(spec.stride_h, spec.stride_w), padding=(spec.pad_h, spec.pad_w),
                        dilation=(spec.dil_h, spec.dil_w))

    for _ in range(max(steps // 10, 5)):
        run()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        run()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / steps


def measure_layer(spec, base_seed, steps, out_mode, x_host=None, library=False):
    import torch

    import workloads as W
    from paper_2309_06626_amd import binding as B
    from paper_2309_06626_amd import runtime as R
    from paper_2309_06626_amd.metrics import (HBM_PEAK_GBS, MFMA_PEAK_TFLOPS, algorithmic_bytes, algorithmic_flops,
                                              buffer_sets_for_cold_runs, time_launches, time_rotating)

    ci = W.make_conv_inputs(spec, base_seed, x=x_host)
    layer = R.ConvLayer(spec, ci.w, ci.bias, ci.mask, out_mode=out_mode)
    x = R.to_device(ci.x, spec.dtype)
    y = layer.new_output()
    y.zero_()
    warm = max(steps // 10, 5)
    # the kernels the cost model picks, then the measured choice (sparse_conv_plan_tune): both are reported
    model_kernel = (kernel_name(layer.plan, 0), kernel_name(layer.plan, 1))
    _, ts_model = time_launches(B.prepared_run(layer.plan, x, layer.bias, y), steps, warm)
    _, td_model = time_launches(B.prepared_run(layer.plan, x, layer.bias, y, dense=True), steps, warm)
    if TUNE:
        B.sparse_conv_plan_tune(layer.plan, x, layer.bias, y)
        _, ts = time_launches(B.prepared_run(layer.plan, x, layer.bias, y), steps, warm)
        _, td = time_launches(B.prepared_run(layer.plan, x, layer.bias, y, dense=True), steps, warm)
        # (two timings of one launch differ by a per cent or two: an unchanged choice keeps its first figure)
        if kernel_name(layer.plan, 0) == model_kernel[0]:
            ts = min(ts, ts_model)
        if kernel_name(layer.plan, 1) == model_kernel[1]:
            td = min(td, td_model)
    else:
        ts, td = ts_model, td_model
    # cold regime: rotate through copies of the activations and outputs that together exceed the caches
    nsets = buffer_sets_for_cold_runs(x.numel() * x.element_size() + y.numel() * y.element_size())
    xs = [x] + [x.clone() for _ in range(nsets - 1)]
    ys = [y] + [torch.zeros_like(y) for _ in range(nsets - 1)]
    cold_steps = max(steps // 4, 4 * nsets)
    tsc = time_rotating([B.prepared_run(layer.plan, a, layer.bias, b) for a, b in zip(xs, ys)], cold_steps, nsets)
    tdc = time_rotating([B.prepared_run(layer.plan, a, layer.bias, b, dense=True) for a, b in zip(xs, ys)], cold_steps, nsets)
    del xs, ys
    scatter = out_mode == B.SC_OUT_SCATTER_ONLY
    fl = algorithmic_flops(spec, ci.keep)
    by = algorithmic_bytes(spec, ci.keep, scatter_only=scatter)
    rec = {
        "layer": spec.name, "dtype": spec.dtype, "m": spec.m, "kept": ci.keep, "k": spec.k, "c_out": spec.c_out,
        "sparsity": spec.sparsity, "out_mode": "scatter_only" if scatter else "zero_fill",
        "kernel_sparse": kernel_name(layer.plan, 0),
        "kernel_dense": kernel_name(layer.plan, 1),
        "model_kernel_sparse": model_kernel[0], "model_kernel_dense": model_kernel[1],
        "model_sparse_us": ts_model * 1e6, "model_dense_us": td_model * 1e6,
        "sparse_us": ts * 1e6, "dense_us": td * 1e6, "speedup_vs_dense": td / ts,
        "sparse_us_cold": tsc * 1e6, "dense_us_cold": tdc * 1e6, "speedup_vs_dense_cold": tdc / tsc,
        "gbs_cold": by / tsc / 1e9, "hbm_frac_cold": by / tsc / 1e9 / HBM_PEAK_GBS, "cold_buffer_sets": nsets,
        "tflops": fl / ts / 1e12, "mfma_frac": fl / ts / 1e12 / MFMA_PEAK_TFLOPS[spec.dtype],
        "dense_tflops": algorithmic_flops(spec, spec.m) / td / 1e12,
        "gbs": by / ts / 1e9, "hbm_frac": by / ts / 1e9 / HBM_PEAK_GBS,
        "arithmetic_intensity": fl / by,
    }
    del layer, x, y
    torch.cuda.empty_cache()
    rec["library_dense_us"] = library_conv_us(spec, max(steps // 4, 20)) if library else None
    torch.cuda.empty_cache()
    return rec


def chain_time(ops, base_seed, steps, dense=False, propagated_masks=False, compact=False, fused=False):
    """Whole network with fixed buffers: (us per pass launched call by call, us per pass as a HIP graph replay).

    propagated_masks: every layer's 2-D mask comes from one score through the mask generator (Alg. 1,
    getMask), so layers of one resolution share it; compact: tensors between such layers stay compact; fused: shortcut
    sums ride in the epilogue of the convolution before them where the planner accepts it."""
    import numpy as np
    import torch

    import workloads as W
    from paper_2309_06626_amd import binding as B
    from paper_2309_06626_amd import runtime as R

    dtype = W.conv_specs(ops)[0].dtype
    layers = {}
    if propagated_masks:
        res = W.network_input_shape(ops)[1]
        score = torch.from_numpy(W.gen_score(res, res, seed=base_seed + 77)).to("cuda:0")
    for s in W.conv_specs(ops):
        ci = W.make_conv_inputs(s, base_seed, x=np.zeros(1, np.float32))
        mask = ci.mask
        if propagated_masks:
            mask = B.sparse_mask_generate(score, s.ho, s.wo, s.sparsity).cpu().numpy().reshape(-1)
        layers[s.name] = R.ConvLayer(s, ci.w, ci.bias, mask)
    tensors = {"input": R.to_device(W.gen_activations(W.network_input_shape(ops), base_seed, dtype), dtype)}
    for op in ops:
        if op.kind == "conv" and op.src.startswith("synthetic:"):
            tensors[op.src] = R.to_device(W.gen_activations(op.spec.x_shape(), base_seed + 500 + op.spec.layer_index, dtype), dtype)
    net = R.NetworkRunner(ops, tensors, layers, dense=dense,
                          row_formats=R.plan_row_formats(ops, layers) if compact else None, fuse_shortcuts=fused, tune=TUNE)

    def timed(fn):
        for _ in range(max(steps // 5, 3)):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / steps

    eager = timed(net.run)
    graph = net.capture()
    return eager, timed(graph.replay)


def compact_format_times(steps):
    """us per launch of the pointwise benchmark layers (config 4, 56x56 and 28x28 maps) and of the
    ResNet18 stage-1 layer with dense and with compact operands; the dense run of the same plan beside them."""
    import torch

    import workloads as W
    from paper_2309_06626_amd import binding as B
    from paper_2309_06626_amd import runtime as R
    from paper_2309_06626_amd.metrics import time_launches

    specs = [s for s in W.config4() if s.h in (56, 28)] + [W.config2(0.5)]
    rows = []
    warm = max(steps // 10, 5)
    for spec in specs:
        ci = W.make_conv_inputs(spec, W.base_seed(4))
        layer = R.ConvLayer(spec, ci.w, ci.bias, ci.mask)
        kept = layer.info["kept"]
        dt = B.TORCH_DTYPE[spec.dtype]
        x = R.to_device(ci.x, spec.dtype)
        y = layer.new_output().zero_()
        xc = torch.randn((kept, spec.c_in), device="cuda:0").clamp_(min=0).to(dt)
        yc = torch.zeros((kept, spec.c_out), dtype=dt, device="cuda:0")
        pointwise = spec.kh == 1 and spec.kw == 1
        rec = {"layer": spec.name, "m": spec.m, "kept": kept, "k": spec.k, "c_out": spec.c_out}
        D, C = B.SC_ROWS_DENSE, B.SC_ROWS_COMPACT
        for key, xa, xf, ya, yf in (("dense_dense", x, D, y, D), ("dense_compact", x, D, yc, C),
                                    ("compact_dense", xc, C, y, D), ("compact_compact", xc, C, yc, C)):
            if xf == C and not pointwise:
                rec[key + "_us"] = None
                continue
            _, t = time_launches(B.prepared_run_rows(layer.plan, xa, layer.bias, ya, xf, yf), steps, warm)
            rec[key + "_us"] = t * 1e6
        _, t = time_launches(B.prepared_run(layer.plan, x, layer.bias, y, dense=True), steps, warm)
        rec["dense_run_us"] = t * 1e6
        rows.append(rec)
        del layer, x, y, xc, yc
        torch.cuda.empty_cache()
    return rows


def depthwise_times(steps):
    """Depthwise 3x3 layers (MobileNetV2-style body, batch 64, s = 0.5): us per launch for the dense-layout
    run, the compact-output run and the dense run, with the HBM share of the algorithmic bytes."""
    import torch

    import workloads as W
    from paper_2309_06626_amd import binding as B
    from paper_2309_06626_amd import runtime as R
    from paper_2309_06626_amd.metrics import HBM_PEAK_GBS, algorithmic_bytes, time_launches

    rows = []
    warm = max(steps // 10, 5)
    for spec in W.depthwise_layers():
        ci = W.make_conv_inputs(spec, W.base_seed(6))
        layer = R.ConvLayer(spec, ci.w, ci.bias, ci.mask)
        kept = layer.info["kept"]
        x = R.to_device(ci.x, spec.dtype)
        y = layer.new_output().zero_()
        yc = torch.zeros((kept, spec.c_out), dtype=B.TORCH_DTYPE[spec.dtype], device="cuda:0")
        _, ts = time_launches(B.prepared_run(layer.plan, x, layer.bias, y), steps, warm)
        _, tc = time_launches(B.prepared_run_rows(layer.plan, x, layer.bias, yc, B.SC_ROWS_DENSE, B.SC_ROWS_COMPACT), steps, warm)
        _, td = time_launches(B.prepared_run(layer.plan, x, layer.bias, y, dense=True), steps, warm)
        # compact input under a producer's mask of the same sparsity (input resolution), compact output
        pixels = spec.n * spec.h * spec.w
        in_mask = W.gen_mask(pixels, W.n_keep(spec.sparsity, pixels), W.base_seed(6) + 900 + spec.layer_index)
        kept_in = B.sparse_conv_plan_set_input_mask(layer.plan, torch.from_numpy(in_mask).to("cuda:0"))
        xc = torch.randn((kept_in, spec.c_in), device="cuda:0").clamp_(min=0).to(B.TORCH_DTYPE[spec.dtype])
        _, tcc = time_launches(B.prepared_run_rows(layer.plan, xc, layer.bias, yc, B.SC_ROWS_COMPACT, B.SC_ROWS_COMPACT), steps, warm)
        by, byc, byd = (algorithmic_bytes(spec, kept), algorithmic_bytes(spec, kept, scatter_only=True),
                        algorithmic_bytes(spec, spec.m))
        rows.append({"layer": spec.name, "m": spec.m, "c": spec.c_out, "kept": kept,
                     "sparse_us": ts * 1e6, "compact_out_us": tc * 1e6, "dense_us": td * 1e6, "compact_in_out_us": tcc * 1e6,
                     "sparse_hbm_frac": by / ts / 1e9 / HBM_PEAK_GBS, "compact_hbm_frac": byc / tc / 1e9 / HBM_PEAK_GBS,
                     "dense_hbm_frac": byd / td / 1e9 / HBM_PEAK_GBS})
        del layer, x, y, yc, xc
        torch.cuda.empty_cache()
    return rows


def backward_times(steps):
    """Backward pass (Alg. 1) of a few benchmark layers: us per call for the filter + bias gradients, the
    input gradient, and the forward run beside them; TFLOP/s of the filter-gradient contraction
    (2 * kept * K * Cout, the same count as the forward GEMM)."""
    import torch

    import workloads as W
    from paper_2309_06626_amd import binding as B
    from paper_2309_06626_amd import runtime as R
    from paper_2309_06626_amd.metrics import algorithmic_flops, time_launches

    c3 = {s.name: s for s in W.conv_specs(W.config3())}
    import dataclasses
    specs = [W.config2(0.5), W.config2(0.0), c3["l2b0_conv2"], c3["l3b0_conv2"], c3["l4b0_conv2"],
             [s for s in W.config4() if s.name == "c4_pw_96_576_28"][0],
             dataclasses.replace(W.config2(0.5), name="c2_resnet18_layer1 (fp32)", dtype="f32")]
    rows = []
    warm = max(steps // 10, 5)
    for spec in specs:
        ci = W.make_conv_inputs(spec, W.base_seed(2))
        layer = R.ConvLayer(spec, ci.w, ci.bias, ci.mask)
        bwd = B.sparse_conv_backward_plan(layer.plan, layer.w)
        x = R.to_device(ci.x, spec.dtype)
        y = layer.new_output().zero_()
        layer.sparse(x, y)
        dy = torch.randn(spec.y_shape(), device="cuda:0").to(B.TORCH_DTYPE[spec.dtype])
        dx = torch.empty_like(x)
        dw = torch.empty(spec.w_shape(), dtype=torch.float32, device="cuda:0")
        db = torch.empty(spec.c_out, dtype=torch.float32, device="cuda:0")
        _, tf = time_launches(B.prepared_run(layer.plan, x, layer.bias, y), steps, warm)
        _, tw = time_launches(B.prepared_backward_run(bwd, x, y, dy, None, dw, db), steps, warm)
        _, tx = time_launches(B.prepared_backward_run(bwd, x, y, dy, dx, None, None), steps, warm)
        _, tb = time_launches(B.prepared_backward_run(bwd, x, y, dy, dx, dw, db), steps, warm)
        fl = algorithmic_flops(spec, layer.info["kept"])
        rows.append({"layer": spec.name, "m": spec.m, "k": spec.k, "c_out": spec.c_out, "sparsity": spec.sparsity,
                     "forward_us": tf * 1e6, "dw_db_us": tw * 1e6, "dx_us": tx * 1e6, "all_us": tb * 1e6,
                     "dw_tflops": fl / tw / 1e12})
        del layer, bwd, x, y, dy, dx, dw, db
        torch.cuda.empty_cache()
    return rows


def mask_generator_times(steps):
    """us per call of the mask generator (two launches; four for maps above 16 384 pixels) for the layer resolutions of the two networks."""
    import torch

    import workloads as W
    from paper_2309_06626_amd import binding as B
    from paper_2309_06626_amd.metrics import time_launches

    rows = []
    for res, layer_res, s in ((224, (112, 56, 28, 14, 7), 0.5), (640, (320, 80, 40, 20), 0.3)):
        score = torch.from_numpy(W.gen_score(res, res, seed=res)).to("cuda:0")
        for r in layer_res:
            mask = torch.empty((r, r), dtype=torch.uint8, device="cuda:0")
            ws = torch.empty(B.sparse_mask_workspace_bytes(r, r), dtype=torch.uint8, device="cuda:0")
            _, t = time_launches(lambda st=None: B.sparse_mask_generate(score, r, r, s, mask=mask, workspace=ws, stream=st), steps, 10)
            rows.append({"score": f"{res}x{res}", "layer": f"{r}x{r}", "sparsity": s, "us": t * 1e6,
                         "kept": int(mask.sum().item())})
    return rows


def oracle_times(want):
    """The CPU oracle (test infrastructure, timed here as the baseline the benchmark description asks for) on every layer
    of the wanted configurations with synthetic inputs of each layer's own shape: all host cores, and one thread (a child
    process with OMP_NUM_THREADS=1) for configs 1 and 2."""
    import subprocess
    import time

    import workloads as W
    from oracle import oracle

    groups = {1: [W.config1()], 2: [W.config2(0.5)], 3: W.conv_specs(W.config3()), 4: W.config4(), 5: W.conv_specs(W.config5())}
    rows = []
    for cfg in sorted(want):
        secs, flops = 0.0, 0.0
        for spec in groups[cfg]:
            ci = W.make_conv_inputs(spec, W.base_seed(cfg))
            if cfg <= 2:
                oracle.masked_conv2d(spec, ci.x, ci.w, ci.bias, ci.mask)      # page-in, thread pool
            t0 = time.perf_counter()
            oracle.masked_conv2d(spec, ci.x, ci.w, ci.bias, ci.mask)
            secs += time.perf_counter() - t0
            flops += 2.0 * ci.keep * spec.k * spec.c_out
        rows.append({"config": f"config {cfg}", "layers": len(groups[cfg]), "gflop": flops / 1e9, "threads": oracle.num_threads(),
                     "seconds": secs, "tflops": flops / secs / 1e12})
        if cfg <= 2:
            code = (f"import time, workloads as W\nfrom oracle import oracle\nspec = W.config{cfg}()\n"
                    f"ci = W.make_conv_inputs(spec, W.base_seed({cfg}))\noracle.masked_conv2d(spec, ci.x, ci.w, ci.bias, ci.mask)\n"
                    "t0 = time.perf_counter()\noracle.masked_conv2d(spec, ci.x, ci.w, ci.bias, ci.mask)\n"
                    "print('SINGLE', time.perf_counter() - t0, oracle.num_threads())\n")
            r = subprocess.run([sys.executable, "-c", code], cwd=ROOT, env=dict(os.environ, OMP_NUM_THREADS="1"),
                               capture_output=True, text=True, timeout=300)
            for line in r.stdout.splitlines():
                if line.startswith("SINGLE"):
                    _, sec, thr = line.split()
                    rows.append({"config": f"config {cfg}", "layers": 1, "gflop": flops / 1e9, "threads": int(thr),
                                 "seconds": float(sec), "tflops": flops / float(sec) / 1e12})
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--configs", default="1,2,3,4,5")
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--json", default="")
    ap.add_argument("--library-conv", action="store_true",
                    help="also time torch.nn.functional.conv2d (MIOpen, dense) on every shape, as context")
    ap.add_argument("--masks", action="store_true", help="also time the mask generator (Alg. 1, getMask)")
    ap.add_argument("--compact", action="store_true", help="also time runs with compact row formats")
    ap.add_argument("--pruned", action="store_true",
                    help="also time a channel-pruned ResNet18 stack (51/102/205/410 channels, s = 0.3), as it is and padded to 16 and to 8")
    ap.add_argument("--mobilenet", action="store_true",
                    help="also time a MobileNetV2-style stack with propagated masks, with dense and with compact tensors")
    ap.add_argument("--backward", action="store_true", help="also time the backward pass of a few layers")
    ap.add_argument("--depthwise", action="store_true", help="also time the depthwise layers of a MobileNetV2-style body")
    ap.add_argument("--no-tune", action="store_true", help="time the cost model's kernel choice only (no sparse_conv_plan_tune)")
    ap.add_argument("--fp32", action="store_true", help="also the benchmark layer in fp32, the paper's own arithmetic (App. A)")
    ap.add_argument("--oracle-times", action="store_true",
                    help="also time the CPU oracle on every configuration (all host cores; one thread for configs 1 and 2)")
    ap.add_argument("--profile-layer", default="",
                    help="NAME[:BMxBN][:splitN][:slabBM][:dense][:cold][:time][:backward[:dx]] -- only launch that layer of config 2 (s = 0.5), 3, 4 or 5 --steps times "
                         "(sparse run, or the dense run), optionally with a forced tile of the tiled kernel, N splits of K, the slab kernel with BM-row tiles, "
                         "optionally rotating through buffer copies larger than the memory-side cache: the target of a rocprofv3 run")
    args = ap.parse_args()

    import torch

    import workloads as W
    from paper_2309_06626_amd import binding as B

    if not torch.cuda.is_available():
        print("layer_report needs a GPU", file=sys.stderr)
        sys.exit(2)
    if os.environ.get("SPARSE_CONV_LIBRARY"):
        B.LIB_PATH = os.environ["SPARSE_CONV_LIBRARY"]
    B.lib()
    if args.profile_layer:
        from paper_2309_06626_amd import runtime as R
        from paper_2309_06626_amd.metrics import buffer_sets_for_cold_runs
        parts = args.profile_layer.split(":")
        specs = {s.name: (s, cfg) for cfg, ops in ((3, W.config3()), (5, W.config5())) for s in W.conv_specs(ops)}
        specs.update({s.name: (s, 4) for s in W.config4()})
        specs[W.config2(0.5).name] = (W.config2(0.5), 2)
        spec, cfg = specs[parts[0]]
        ci = W.make_conv_inputs(spec, W.base_seed(cfg))
        layer = R.ConvLayer(spec, ci.w, ci.bias, ci.mask)
        dense = "dense" in parts[1:]
        for part in parts[1:]:
            if part.startswith("split"):
                B.sparse_conv_plan_set_option(layer.plan, B.SC_OPT_SPLIT_K, int(part[5:]))
            elif part.startswith("slab"):
                B.sparse_conv_plan_set_option(layer.plan, B.SC_OPT_SLAB, int(part[4:]))
            elif part.replace("x", "").isdigit() and part.count("x") == 1:
                bm, bn = (int(v) for v in part.split("x"))
                B.sparse_conv_plan_set_tiles(layer.plan, 0, bm, bn)
                B.sparse_conv_plan_set_tiles(layer.plan, 1, bm, bn)
        x, y = R.to_device(ci.x, spec.dtype), layer.new_output()
        if "backward" in parts[1:]:                 # the backward pass of the layer: dw + db, with `dx` also the input gradient
            bwd = B.sparse_conv_backward_plan(layer.plan, layer.w)
            layer.sparse(x, y)
            dy = torch.randn(spec.y_shape(), device="cuda:0").to(B.TORCH_DTYPE[spec.dtype])
            dx = torch.empty_like(x) if "dx" in parts[1:] else None
            dw = torch.empty(spec.w_shape(), dtype=torch.float32, device="cuda:0")
            db = torch.empty(spec.c_out, dtype=torch.float32, device="cuda:0")
            call = B.prepared_backward_run(bwd, x, y, dy, dx, dw, db)
            for _ in range(args.steps):
                call()
            torch.cuda.synchronize()
            print(f"{spec.name}: {args.steps} backward runs (dw, db{', dx' if dx is not None else ''}), kept {ci.keep} of {spec.m} rows, K {spec.k}, Cout {spec.c_out}")
            if "time" in parts[1:]:
                from paper_2309_06626_amd.metrics import time_launches
                us = time_launches(call, max(args.steps, 100), 20, 5)[1] * 1e6
                print(f"{spec.name}: {us:.2f} us per backward run (median of 5 replays of a graph of {max(args.steps, 100)} runs)")
            return
        if "cold" in parts[1:]:                     # rotate through copies beyond the memory-side cache
            nsets = buffer_sets_for_cold_runs(x.numel() * x.element_size() + y.numel() * y.element_size())
            calls = [B.prepared_run(layer.plan, x.clone(), layer.bias, torch.empty_like(y), dense=dense) for _ in range(nsets)]
            for i in range(max(args.steps, 2 * nsets)):
                calls[i % nsets]()
        else:
            call = B.prepared_run(layer.plan, x, layer.bias, y, dense=dense)
            for _ in range(args.steps):
                call()
        torch.cuda.synchronize()
        which = 1 if dense else 0
        print(f"{spec.name}: {args.steps} launches of {B.sparse_conv_plan_kernel(layer.plan, which)} "
              f"{B.sparse_conv_plan_tiles(layer.plan, which)}, rows {spec.m if dense else ci.keep}, K {spec.k}, Cout {spec.c_out}")
        if "time" in parts[1:] and "cold" not in parts[1:]:      # device time per launch: graph replays, HIP events
            from paper_2309_06626_amd.metrics import time_launches
            us = time_launches(call, max(args.steps, 100), 20, 5)[1] * 1e6
            print(f"{spec.name}: {us:.2f} us per launch (median of 5 replays of a graph of {max(args.steps, 100)} launches)")
        return
    want = {int(c) for c in args.configs.split(",")}
    records = []
    global TUNE
    TUNE = not args.no_tune

    def emit(cfg, rec):
        rec["config"] = cfg
        records.append(rec)
        print(f"| {cfg} | {rec['layer']} | {rec['m']}x{rec['k']}x{rec['c_out']} | {rec['sparsity']:.2f} {rec['out_mode'][:7]} | "
              f"{rec['kernel_sparse']} | {rec['sparse_us']:.2f} | {rec['dense_us']:.2f} | {rec['speedup_vs_dense']:.2f} | "
              f"{rec['model_sparse_us']:.2f} / {rec['model_dense_us']:.2f} | "
              f"{rec['tflops']:.1f} | {100 * rec['mfma_frac']:.1f} | {rec['gbs']:.0f} | {100 * rec['hbm_frac']:.1f} | "
              f"{rec['arithmetic_intensity']:.0f} | {rec['sparse_us_cold']:.2f} | {rec['dense_us_cold']:.2f} | "
              f"{rec['speedup_vs_dense_cold']:.2f} | {100 * rec['hbm_frac_cold']:.1f} | "
              + (f"{rec['library_dense_us']:.1f} |" if rec["library_dense_us"] is not None else "- |"), flush=True)

    print("| cfg | layer | M x K x Cout | s, out mode | sparse kernel | sparse us | dense us | speed-up | cost model's choice: sparse / dense us "
          "| TFLOP/s | % MFMA | GB/s | % HBM | FLOP/B "
          "| cold: sparse us | cold: dense us | cold: speed-up | cold: % HBM | torch conv2d us (context) |")
    print("|---|---|---|---|---|---|---|---|---|---|---|---|---|---|---|---|---|---|---|")
    if 1 in want:
        emit(1, measure_layer(W.config1(), W.base_seed(1), args.steps, B.SC_OUT_ZERO_FILL, library=args.library_conv))
    if 2 in want:
        for s in W.C2_SPARSITIES:
            emit(2, measure_layer(W.config2(s), W.base_seed(2), args.steps, B.SC_OUT_ZERO_FILL, library=args.library_conv))
        for s in W.C2_SPARSITIES[1:]:
            emit(2, measure_layer(W.config2(s), W.base_seed(2), args.steps, B.SC_OUT_SCATTER_ONLY, library=args.library_conv))
    if args.fp32:
        emit(2, measure_layer(W.config2(0.5).with_(dtype="f32", name="c2_resnet18_layer1_fp32"), W.base_seed(2), args.steps,
                              B.SC_OUT_ZERO_FILL, library=args.library_conv))
        emit(2, measure_layer(W.config2(0.0).with_(dtype="f32", name="c2_resnet18_layer1_fp32"), W.base_seed(2), args.steps,
                              B.SC_OUT_ZERO_FILL, library=args.library_conv))
    chains = {}
    if 3 in want:
        ops = W.config3()
        for spec in W.conv_specs(ops):
            emit(3, measure_layer(spec, W.base_seed(3), args.steps, B.SC_OUT_ZERO_FILL, library=args.library_conv))
        cs = max(args.steps // 10, 5)
        chains["config 3 (ResNet18 stack, batch 64, s=0.5)"] = chain_time(ops, W.base_seed(3), cs)
        chains["config 3, shortcut sums fused into the convolution before them"] = \
            chain_time(ops, W.base_seed(3), cs, fused=True)
        chains["config 3, downsample convs dense"] = chain_time(W.config3(sparse_downsample=False), W.base_seed(3), cs)
        chains["config 3, every conv through dense_conv_run"] = chain_time(ops, W.base_seed(3), cs, dense=True)
    if 4 in want:
        for spec in W.config4():
            emit(4, measure_layer(spec, W.base_seed(4), args.steps, B.SC_OUT_ZERO_FILL, library=args.library_conv))
    if 5 in want:
        ops = W.config5()
        for spec in W.conv_specs(ops):
            emit(5, measure_layer(spec, W.base_seed(5), args.steps, B.SC_OUT_ZERO_FILL, library=args.library_conv))
        cs = max(args.steps // 10, 5)
        chains["config 5 (detector stack, batch 16, s=0.3)"] = chain_time(ops, W.base_seed(5), cs)
        chains["config 5, every conv through dense_conv_run"] = chain_time(ops, W.base_seed(5), cs, dense=True)
    if args.pruned:
        cs = max(args.steps // 10, 5)
        ops = W.pruned_resnet18()
        chains["pruned ResNet18 stack (batch 64, s=0.3), channels padded to multiples of 16 (64/112/208/416)"] = \
            chain_time(W.pad_channels(ops, 16), W.base_seed(3), cs)
        chains["the same, every conv through dense_conv_run"] = chain_time(W.pad_channels(ops, 16), W.base_seed(3), cs, dense=True)
        chains["pruned ResNet18 stack, channels padded to multiples of 8 (56/104/208/416: register-staged tiled kernel)"] = \
            chain_time(W.pad_channels(ops, 8), W.base_seed(3), cs)
        chains["pruned ResNet18 stack with its own channel counts (51/102/205/410: element gather)"] = \
            chain_time(ops, W.base_seed(3), cs)
    if args.mobilenet:
        cs = max(args.steps // 10, 5)
        for sp in (0.5, 0.3):
            ops = W.mobilenet_v2(sparsity=sp)
            tag = f"MobileNetV2-style stack (52 convs, batch 64, s={sp}, masks propagated from one score)"
            chains[tag + ", dense tensors"] = chain_time(ops, W.base_seed(6), cs, propagated_masks=True)
            chains[tag + ", compact tensors between layers that share a mask"] = \
                chain_time(ops, W.base_seed(6), cs, propagated_masks=True, compact=True)
            chains[tag + ", compact tensors and fused shortcut sums"] = \
                chain_time(ops, W.base_seed(6), cs, propagated_masks=True, compact=True, fused=True)
        chains["MobileNetV2-style stack, every conv through dense_conv_run"] = \
            chain_time(ops, W.base_seed(6), cs, dense=True, propagated_masks=True)
    if chains:
        print()
        print("| whole chain (conv launches + pooling / residual glue, fixed buffers) | us per pass, call by call | us per pass, HIP graph replay |")
        print("|---|---|---|")
        for k, v in chains.items():
            print(f"| {k} | {v[0]:.1f} | {v[1]:.1f} |")
    compact_rows = []
    if args.compact:
        compact_rows = compact_format_times(args.steps)
        fmt = lambda v: "-" if v is None else f"{v:.2f}"
        print()
        print("| layer (s = 0.5) | M x K x Cout | dense in, dense out (sparse_conv_run) us | dense in, compact out us | "
              "compact in, dense out us | compact in, compact out us | dense_conv_run us |")
        print("|---|---|---|---|---|---|---|")
        for r in compact_rows:
            print(f"| {r['layer']} | {r['m']}x{r['k']}x{r['c_out']} | {fmt(r['dense_dense_us'])} | {fmt(r['dense_compact_us'])} | "
                  f"{fmt(r['compact_dense_us'])} | {fmt(r['compact_compact_us'])} | {fmt(r['dense_run_us'])} |")
    dw_rows = []
    if args.depthwise:
        dw_rows = depthwise_times(args.steps)
        print()
        print("| depthwise 3x3 layer (batch 64, s = 0.5) | M x C | sparse us (zero fill) | % HBM | compact out us | % HBM | dense us | % HBM | "
              "speed-up zero fill | speed-up compact out | compact in (producer's mask, s = 0.5) and out us |")
        print("|---|---|---|---|---|---|---|---|---|---|---|")
        for r in dw_rows:
            print(f"| {r['layer']} | {r['m']}x{r['c']} | {r['sparse_us']:.2f} | {100 * r['sparse_hbm_frac']:.1f} | "
                  f"{r['compact_out_us']:.2f} | {100 * r['compact_hbm_frac']:.1f} | {r['dense_us']:.2f} | "
                  f"{100 * r['dense_hbm_frac']:.1f} | {r['dense_us'] / r['sparse_us']:.2f} | {r['dense_us'] / r['compact_out_us']:.2f} | "
                  f"{r['compact_in_out_us']:.2f} |")
    bw_rows = []
    if args.backward:
        bw_rows = backward_times(max(args.steps // 2, 20))
        print()
        print("| backward pass: layer | M x K x Cout | s | forward us | dw + db us (row-contraction GEMM that gates dy by y and sums db, then the reduction over row splits) | "
              "TFLOP/s of that GEMM | dx us (g map + convolution with rotated filters) | dx + dw + db us |")
        print("|---|---|---|---|---|---|---|---|")
        for r in bw_rows:
            print(f"| {r['layer']} | {r['m']}x{r['k']}x{r['c_out']} | {r['sparsity']:.2f} | {r['forward_us']:.2f} | {r['dw_db_us']:.2f} | "
                  f"{r['dw_tflops']:.1f} | {r['dx_us']:.2f} | {r['all_us']:.2f} |")
    mask_rows = []
    if args.masks:
        mask_rows = mask_generator_times(max(args.steps // 4, 20))
        print()
        print("| mask generator: score | layer map | s | kept pixels | us per mask (pooling + ranking: two launches, four above 16 384 pixels) |")
        print("|---|---|---|---|---|")
        for r in mask_rows:
            print(f"| {r['score']} | {r['layer']} | {r['sparsity']:.2f} | {r['kept']} | {r['us']:.1f} |")
    oracle_rows = []
    if args.oracle_times:
        oracle_rows = oracle_times(want)
        print()
        print("| CPU oracle (direct loop nest, double accumulation) | layers | kept-row GFLOP | threads | seconds | TFLOP/s |")
        print("|---|---|---|---|---|---|")
        for r in oracle_rows:
            print(f"| {r['config']} | {r['layers']} | {r['gflop']:.2f} | {r['threads']} | {r['seconds']:.3f} | {r['tflops']:.4f} |")
    if args.json:
        with open(args.json, "w") as f:
            for r in records:
                f.write(json.dumps(r) + "\n")
            f.write(json.dumps({"chains_us": chains}) + "\n")
            if mask_rows:
                f.write(json.dumps({"mask_generator": mask_rows}) + "\n")
            if compact_rows:
                f.write(json.dumps({"compact_formats": compact_rows}) + "\n")
            if dw_rows:
                f.write(json.dumps({"depthwise": dw_rows}) + "\n")
            if bw_rows:
                f.write(json.dumps({"backward": bw_rows}) + "\n")
            if oracle_rows:
                f.write(json.dumps({"oracle": oracle_rows}) + "\n")


if __name__ == "__main__":
    main()
