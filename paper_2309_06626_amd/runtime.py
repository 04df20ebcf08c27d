"""Tensor marshalling and layer / network drivers on top of the C-ABI binding.

Nothing here computes: host arrays are encoded and copied to the device, the library is
called, results are copied back.
"""
from __future__ import annotations

import hashlib
from typing import Callable, Dict, List, Optional

import numpy as np
import torch

from . import binding as B


def to_device(values_f32: np.ndarray, dtype: str, device="cuda:0") -> torch.Tensor:
    """Host float32 values (already representable in `dtype`) -> device tensor of `dtype`."""
    t = torch.from_numpy(np.ascontiguousarray(values_f32, dtype=np.float32))
    return t.to(B.TORCH_DTYPE[dtype]).to(device).contiguous()


def to_host_f32(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy()


def bits_of(t: torch.Tensor) -> np.ndarray:
    """Raw bit patterns of a device tensor (uint16 / uint32) on the host."""
    view = {2: torch.int16, 4: torch.int32}[t.element_size()]
    a = t.detach().contiguous().view(view).cpu().numpy()
    return a.view({2: np.uint16, 4: np.uint32}[t.element_size()])


class ConvLayer:
    """One planned layer: device filters/bias/mask, workspace, plan handle, output buffer."""

    def __init__(self, spec, w: np.ndarray, bias: Optional[np.ndarray], mask: np.ndarray, device="cuda:0",
                 out_mode=B.SC_OUT_ZERO_FILL, check_count=True):
        self.spec = spec
        self.device = device
        self.w = to_device(w, spec.dtype, device)
        self.bias = torch.from_numpy(np.ascontiguousarray(bias, np.float32)).to(device) if spec.has_bias else None
        self.mask = torch.from_numpy(np.ascontiguousarray(mask, np.uint8)).to(device)
        # identifies the set of kept rows: two layers with equal keys have the same row list
        self.rows_key = (spec.n, spec.ho, spec.wo, spec.mask_mode,
                         hashlib.sha1(np.ascontiguousarray(mask, np.uint8).tobytes()).hexdigest())
        self.desc = B.desc_from_spec(spec, out_mode=out_mode, check_count=check_count)
        self.plan = B.sparse_conv_plan(self.desc, self.mask, self.w)
        self.info = B.sparse_conv_plan_info(self.plan)

    def new_output(self, fill_nan: bool = False) -> torch.Tensor:
        y = torch.empty(self.spec.y_shape(), dtype=B.TORCH_DTYPE[self.spec.dtype], device=self.device)
        if fill_nan:
            y.fill_(float("nan"))
        return y

    def sparse(self, x: torch.Tensor, y: Optional[torch.Tensor] = None) -> torch.Tensor:
        y = self.new_output() if y is None else y
        return B.sparse_conv_run(self.plan, x, self.bias, y)

    def dense(self, x: torch.Tensor, y: Optional[torch.Tensor] = None) -> torch.Tensor:
        y = self.new_output() if y is None else y
        return B.dense_conv_run(self.plan, x, self.bias, y)


def pad_conv_params(spec, padded_spec, w: np.ndarray, bias: Optional[np.ndarray]):
    """Filters and bias of `spec` laid out for `padded_spec` (more input / output channels, NHWC): the
    additional filters, filter entries and bias entries are zero."""
    assert spec.layout == "nhwc" and spec.groups == 1
    wp = np.zeros(padded_spec.w_shape(), dtype=np.float32)
    wp[: spec.c_out, :, :, : spec.c_in] = w
    bp = None
    if spec.has_bias:
        bp = np.zeros(padded_spec.c_out, dtype=np.float32)
        bp[: spec.c_out] = bias
    return wp, bp


kCompactDepthwiseInput = 16 << 20     # input elements from which a depthwise layer reads its input in compact form


def plan_row_formats(ops, layers: Dict[str, "ConvLayer"]) -> Dict[str, bool]:
    """Which tensors of a graph can live as compact [kept x C] matrices (True) instead of dense maps.

    Under mask propagation (Alg. 1, getMask) all layers of one resolution share a mask, so a masked conv may
    hand its kept rows straight to a pointwise (1x1, stride 1, no padding) conv with the same mask, through
    element-wise ops whose operands share that row list, without the scatter, zero fill and re-gather in
    between.  A depthwise layer with windows also reads a compact map: it looks every tap up in the row list
    of its input (the producer's mask, whatever its own).  A tensor stays dense when any consumer needs
    neighbours through the lowering (larger windows with one group, pooling, strided 1x1 layers), when masks
    differ, and at the graph's outputs.  Host-side bookkeeping only."""
    consumers: Dict[str, list] = {}
    for op in ops:
        for src in (op.src, op.src2):
            if src:
                consumers.setdefault(src, []).append(op)
    key: Dict[str, object] = {}
    compact: Dict[str, bool] = {}
    for op in ops:
        if op.kind == "conv":
            key[op.out] = layers[op.spec.name].rows_key
            compact[op.out] = op.spec.layout == "nhwc"
        elif op.kind in ("add", "add_relu"):
            same = key.get(op.src) is not None and key.get(op.src) == key.get(op.src2)
            key[op.out] = key.get(op.src) if same else None
            compact[op.out] = same
        else:
            key[op.out] = None
            compact[op.out] = False

    def accepts(op, name) -> bool:
        """May `op` read tensor `name` in compact form?"""
        if op.kind == "conv":
            sp = op.spec
            if sp.layout != "nhwc":
                return False
            if sp.groups > 1 and sp.kh * sp.kw > 1:
                # depthwise with windows: any known row list.  The rank look-ups cost the layer itself a little
                # (one more dependent fetch per tile); what is saved is the producer's zero fill, which outweighs
                # that only on large maps (measured on MI355X: from about 16 M input elements on)
                return key[name] is not None and sp.n * sp.h * sp.w * sp.c_in >= kCompactDepthwiseInput
            pointwise = (sp.kh == 1 and sp.kw == 1 and sp.stride_h == 1 and sp.stride_w == 1 and sp.pad_h == 0 and
                         sp.pad_w == 0 and sp.groups == 1)
            return pointwise and layers[sp.name].rows_key == key[name]
        if op.kind in ("add", "add_relu"):
            return compact[op.out]
        return False

    changed = True
    while changed:
        changed = False
        for op in ops:
            out = op.out
            if not compact[out]:
                continue
            users = consumers.get(out, [])
            ok = bool(users) and all(accepts(u, out) for u in users)
            if ok and op.kind in ("add", "add_relu"):
                ok = compact.get(op.src, False) and compact.get(op.src2, False)
            if not ok:
                compact[out] = False
                changed = True
    return compact


def plan_shortcut_fusions(ops, layers: Dict[str, "ConvLayer"], row_formats: Optional[Dict[str, bool]] = None,
                          dense: bool = False) -> Dict[str, tuple]:
    """Which sums of a graph can ride in the epilogue of the convolution before them.

    Returns {name of the sum's result: (name of the conv layer, name of the other operand, relu after the sum)}.
    A sum is fused into the operand-producing conv that comes last in the op list, if that conv's result feeds
    nothing else, the other operand exists by then, both have the row format of the result, and the layer runs
    in a kernel with a shortcut path anyway (the tiled kernels and the alternating-group band kernel; the other
    band kernels and the row-panel kernel have none and are faster than a tiled kernel plus a saved launch).
    Host-side bookkeeping only."""
    fmt = row_formats or {}
    position = {op.out: i for i, op in enumerate(ops)}
    producer = {op.out: op for op in ops}
    uses: Dict[str, int] = {}
    for op in ops:
        for src in (op.src, op.src2):
            if src:
                uses[src] = uses.get(src, 0) + 1
    fused = {}
    for op in ops:
        if op.kind not in ("add", "add_relu"):
            continue
        best = None
        for mine, other in ((op.src, op.src2), (op.src2, op.src)):
            conv = producer.get(mine)
            if conv is None or conv.kind != "conv" or uses.get(mine, 0) != 1 or conv.spec.groups != 1:
                continue
            if position.get(other, -1) >= position[mine]:
                continue                                   # the other operand is computed later
            if not (fmt.get(mine, False) == fmt.get(other, False) == fmt.get(op.out, False)):
                continue
            plan = layers[conv.spec.name].plan
            plain = B.sparse_conv_plan_kernel(plan, 1 if dense else 0)
            # the fused launch must not be a step down from the plain one: the same band kernel, or a tiled
            # kernel where the plain run takes one too (runs with compact operands always do)
            if not fmt.get(mine, False):
                if plain in ("band", "band_stream", "band_row_segments", "tile_row_panel"):
                    continue
                if plain in ("band_alternating", "band_tap") and B.sparse_conv_plan_fused_kernel(plan, 1 if dense else 0) != plain:
                    continue
            if best is None or position[mine] > position[best[0]]:
                best = (mine, other)
        if best is not None:
            fused[op.out] = (producer[best[0]].spec.name, best[1], op.kind == "add_relu")
    return fused


def run_network(ops, tensors: Dict[str, torch.Tensor], layers: Dict[str, ConvLayer]) -> Dict[str, torch.Tensor]:
    """Interpret a workload op list on the device (conv = sparse_conv_run, plus the glue ops)."""
    t = dict(tensors)
    for op in ops:
        if op.kind == "conv":
            t[op.out] = layers[op.spec.name].sparse(t[op.src])
        elif op.kind == "maxpool":
            t[op.out] = B.sc_maxpool2d_nhwc(t[op.src], 3, 2, 1)
        elif op.kind == "add_relu":
            t[op.out] = B.sc_add_relu(t[op.src], t[op.src2])
        elif op.kind == "add":
            t[op.out] = B.sc_add(t[op.src], t[op.src2])
        else:
            raise ValueError(op.kind)
    return t


class NetworkRunner:
    """A workload op list bound to fixed device buffers: every tensor is allocated once and every
    launch is validated once, so a pass is a plain sequence of C-ABI calls (and can be recorded into
    a HIP graph: the library launches kernels only, no memsets, no allocations, no synchronisation)."""

    def __init__(self, ops, tensors: Dict[str, torch.Tensor], layers: Dict[str, ConvLayer], dense: bool = False,
                 row_formats: Optional[Dict[str, bool]] = None, fuse_shortcuts: bool = False, tune: bool = False):
        """row_formats: the result of plan_row_formats, to keep those tensors compact (sparse runs only).
        fuse_shortcuts: sums that plan_shortcut_fusions accepts run in the epilogue of their conv; the conv's own
        result is then never materialised (its name is absent from the tensors).
        tune: every convolution with dense operands gets its kernels chosen by measurement on the network's own
        buffers (sparse_conv_plan_tune) before the launches are prepared."""
        self.tensors = dict(tensors)
        self.calls: List[Callable] = []
        self.row_formats = {} if (dense or row_formats is None) else dict(row_formats)
        self.fusions = plan_shortcut_fusions(ops, layers, self.row_formats, dense) if fuse_shortcuts else {}
        fused_conv = {v[0]: (k, v[1], v[2]) for k, v in self.fusions.items()}   # conv layer -> (sum, other operand, relu)
        fmt = lambda name: B.SC_ROWS_COMPACT if self.row_formats.get(name, False) else B.SC_ROWS_DENSE
        t = self.tensors
        rows_mask: Dict[str, torch.Tensor] = {}       # the mask whose kept rows a tensor holds when compact
        for op in ops:
            if op.kind != "conv":
                if op.src in rows_mask:
                    rows_mask[op.out] = rows_mask[op.src]
            else:
                rows_mask[op.out] = layers[op.spec.name].mask
        for op in ops:
            if op.kind == "conv" and op.spec.name in fused_conv:
                layer = layers[op.spec.name]
                out, other, relu = fused_conv[op.spec.name]
                xf, yf = fmt(op.src), fmt(out)
                t[out] = torch.empty_like(t[other])
                if tune and xf == B.SC_ROWS_DENSE and yf == B.SC_ROWS_DENSE:
                    # (the measured tile serves the fused launch too; its output buffer is scratch for the measurement)
                    B.sparse_conv_plan_tune(layer.plan, t[op.src], layer.bias, t[out])
                self.calls.append(B.prepared_run_residual(layer.plan, t[op.src], layer.bias, t[other], t[out], relu, xf, yf,
                                                          dense=dense))
                continue
            if op.kind in ("add", "add_relu") and op.out in self.fusions:
                continue
            if op.kind == "conv":
                layer = layers[op.spec.name]
                xf, yf = fmt(op.src), fmt(op.out)
                if xf == B.SC_ROWS_COMPACT and op.spec.groups > 1 and op.spec.kh * op.spec.kw > 1:
                    B.sparse_conv_plan_set_input_mask(layer.plan, rows_mask[op.src])
                if xf == B.SC_ROWS_DENSE and yf == B.SC_ROWS_DENSE:
                    t[op.out] = layer.new_output()
                    if tune:
                        B.sparse_conv_plan_tune(layer.plan, t[op.src], layer.bias, t[op.out])
                    self.calls.append(B.prepared_run(layer.plan, t[op.src], layer.bias, t[op.out], dense=dense))
                    continue
                if yf == B.SC_ROWS_COMPACT:
                    t[op.out] = torch.empty((layer.info["kept"], op.spec.c_out), dtype=B.TORCH_DTYPE[op.spec.dtype],
                                            device=layer.device)
                else:
                    t[op.out] = layer.new_output()
                self.calls.append(B.prepared_run_rows(layer.plan, t[op.src], layer.bias, t[op.out], xf, yf))
            elif op.kind == "maxpool":
                n, h, w, c = t[op.src].shape
                t[op.out] = torch.empty((n, (h + 2 - 3) // 2 + 1, (w + 2 - 3) // 2 + 1, c), dtype=t[op.src].dtype,
                                        device=t[op.src].device)
                self.calls.append(B.prepared_maxpool(t[op.src], t[op.out], 3, 2, 1))
            elif op.kind in ("add", "add_relu"):
                t[op.out] = torch.empty_like(t[op.src])
                self.calls.append(B.prepared_add(t[op.src], t[op.src2], t[op.out], relu=op.kind == "add_relu"))
            else:
                raise ValueError(op.kind)
        self.graph = None

    def run(self, stream_handle=None) -> Dict[str, torch.Tensor]:
        for call in self.calls:
            call(stream_handle)
        return self.tensors

    def capture(self) -> "torch.cuda.CUDAGraph":
        """Record one pass into a HIP graph (replay with .replay()); the buffers stay the same."""
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            self.run(torch.cuda.current_stream().cuda_stream)
        self.graph = g
        return g
