"""Bookkeeping shared by bench.py and layer_report.py: algorithmic work of one layer and launch timing."""
from __future__ import annotations

import time

HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "f16": 2500.0, "f32": 157.3}


def elem_bytes(dtype: str) -> int:
    return 4 if dtype == "f32" else 2


def input_coverage(spec, keep: int) -> float:
    """Fraction of the input pixels that lie inside at least one kept window, for masks that drop a
    uniformly random subset of rows (closed forms for the window shapes of the benchmark networks)."""
    s = 1.0 - keep / spec.m
    kh, st = spec.kh, spec.stride_h
    if kh == 1 and spec.kw == 1:
        return (keep / spec.m) / (st * spec.stride_w)          # exactly the kept pixels
    if kh == 3 and st == 1:
        return 1.0 - s ** 9
    if kh == 3 and st == 2:
        return 1.0 - (s / 4 + s ** 2 / 2 + s ** 4 / 4)
    return 1.0


def algorithmic_bytes(spec, keep: int, scatter_only: bool = False) -> float:
    """Bytes the method itself must move for one launch: the input pixels covered by at least one
    kept window, the filters once, the dense output (zero fill included; kept rows only in
    scatter-only mode), the mask bytes and the row list."""
    eb = elem_bytes(spec.dtype)
    out_rows = keep if scatter_only else spec.m
    # spec.k counts the window entries per output channel (kh*kw for a depthwise layer)
    return (input_coverage(spec, keep) * spec.n * spec.h * spec.w * spec.c_in * eb + spec.k * spec.c_out * eb
            + out_rows * spec.c_out * eb + spec.m + 4 * keep)


def algorithmic_flops(spec, keep: int) -> float:
    return 2.0 * keep * spec.k * spec.c_out


def time_launches(fn, steps: int, warmup: int):
    """(wall seconds, event seconds) per launch of `steps` back-to-back launches on the current stream."""
    import torch

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
    wall = time.perf_counter() - t0
    return wall / steps, e0.elapsed_time(e1) * 1e-3 / steps


def time_rotating(fns, steps: int, warmup: int):
    """Event seconds per launch when the launches cycle through `fns` -- the same operation on different
    buffer sets whose total size exceeds the caches, so every launch finds its operands in HBM only."""
    import torch

    n = len(fns)
    for i in range(warmup):
        fns[i % n]()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(steps):
        fns[i % n]()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e-3 / steps


def buffer_sets_for_cold_runs(bytes_per_set: int, total_bytes: int = 768 << 20, most: int = 64) -> int:
    """Number of (input, output) buffer sets to rotate through so that the sets total more than the
    256 MB memory-side cache plus the L2s by a wide margin."""
    return max(2, min(most, -(-total_bytes // max(bytes_per_set, 1))))
