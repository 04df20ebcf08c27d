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


def warm_clocks(fn, seconds: float = 0.03):
    """Launch for `seconds` before anything is timed: the first launches after an idle period run at ramping clocks, and
    a run of a thousand launches of a few microseconds each would measure mostly that."""
    import torch

    t_end = time.perf_counter() + seconds
    while time.perf_counter() < t_end:
        for _ in range(100):
            fn()
        torch.cuda.synchronize()


class LaunchGraph:
    """`steps` back-to-back launches, cycling through `calls` (callables taking a stream handle), recorded once as a HIP
    graph on a stream of its own and replayed with one host call: device time per launch without the host's launch rate
    in it (layers of a few microseconds are otherwise timed at the speed of the Python loop that launches them)."""

    def __init__(self, calls, steps: int):
        import torch

        self.calls = list(calls) if isinstance(calls, (list, tuple)) else [calls]
        self.steps = steps
        self.stream = torch.cuda.Stream()
        self.graph = torch.cuda.CUDAGraph()
        self.handle = self.stream.cuda_stream
        with torch.cuda.stream(self.stream):
            for c in self.calls:                  # first launches outside the capture (kernel attributes, code load)
                c(self.handle)
            self.stream.synchronize()
            with torch.cuda.graph(self.graph, stream=self.stream):
                for i in range(steps):
                    self.calls[i % len(self.calls)](self.handle)

    def replay(self, warmup: int = 0):
        """(wall seconds, event seconds) of one replay after `warmup` untimed launches."""
        import torch

        with torch.cuda.stream(self.stream):
            for i in range(warmup):
                self.calls[i % len(self.calls)](self.handle)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            self.stream.synchronize()
            t0 = time.perf_counter()
            e0.record(self.stream)
            self.graph.replay()
            e1.record(self.stream)
            self.stream.synchronize()
            wall = time.perf_counter() - t0
        return wall, e0.elapsed_time(e1) * 1e-3


def time_launches(fn, steps: int, warmup: int, repeats: int = 3):
    """(wall seconds, event seconds) per launch: `steps` back-to-back launches replayed as a graph, median of
    `repeats` replays, after the clocks have been warmed up."""
    import statistics

    warm_clocks(fn)
    g = LaunchGraph(fn, steps)
    runs = [g.replay(warmup) for _ in range(repeats)]
    return statistics.median(r[0] for r in runs) / steps, statistics.median(r[1] for r in runs) / steps


def time_rotating(fns, steps: int, warmup: int, repeats: int = 3):
    """Event seconds per launch when the launches cycle through `fns` -- the same operation on different
    buffer sets whose total size exceeds the caches, so every launch finds its operands in HBM only."""
    import statistics

    n = len(fns)
    steps = max(steps, 2 * n)
    warm_clocks(fns[0])
    g = LaunchGraph(fns, steps)
    return statistics.median(g.replay(warmup)[1] for _ in range(repeats)) / steps


def buffer_sets_for_cold_runs(bytes_per_set: int, total_bytes: int = 768 << 20, most: int = 64) -> int:
    """Number of (input, output) buffer sets to rotate through so that the sets total more than the
    256 MB memory-side cache plus the L2s by a wide margin."""
    return max(2, min(most, -(-total_bytes // max(bytes_per_set, 1))))
