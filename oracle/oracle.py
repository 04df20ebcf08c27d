"""Python face of the CPU oracle (TEST INFRASTRUCTURE ONLY).

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py``
may import this module.  It wraps ``masked_conv_oracle.c`` (built with gcc into
``liboracle.so`` beside it) and adds the layer-by-layer interpreter for the small test
networks.  It imports nothing from the HIP package.

Semantics follow the paper's Sec. 3 / Sec. 3.2 / App. A (Alg. 2); see the header of the C
file for every reading taken where the paper is silent.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Dict, List, Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "masked_conv_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O3, OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O3", "-march=x86-64-v2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
               "-ffp-contract=off", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i32p = ctypes.POINTER(ctypes.c_int32)
        i64p = ctypes.POINTER(ctypes.c_int64)
        f32p = ctypes.POINTER(ctypes.c_float)
        f64p = ctypes.POINTER(ctypes.c_double)
        u8p = ctypes.POINTER(ctypes.c_uint8)
        lib.oc_param_count.restype = ctypes.c_int
        lib.oc_num_threads.restype = ctypes.c_int
        lib.oc_out_size.restype = ctypes.c_int
        lib.oc_out_size.argtypes = [ctypes.c_int] * 5
        lib.oc_kept_count.restype = ctypes.c_int64
        lib.oc_kept_count.argtypes = [ctypes.c_double, ctypes.c_int64]
        lib.oc_compact_rows.restype = ctypes.c_int64
        lib.oc_compact_rows.argtypes = [u8p, ctypes.c_int64, i32p]
        lib.oc_masked_conv2d.restype = ctypes.c_int
        lib.oc_masked_conv2d.argtypes = [i32p, f32p, f32p, f32p, u8p, f32p, f64p]
        lib.oc_masked_conv2d_rows.restype = ctypes.c_int
        lib.oc_masked_conv2d_rows.argtypes = [i32p, f32p, f32p, f32p, u8p, i64p, ctypes.c_int64, f32p, f64p]
        lib.oc_masked_conv2d_backward.restype = ctypes.c_int
        lib.oc_masked_conv2d_backward.argtypes = [i32p, f32p, f32p, f32p, f32p, u8p, f64p, f64p, f64p, f64p, f64p]
        lib.oc_round_bf16.restype = None
        lib.oc_round_bf16.argtypes = [f32p, ctypes.c_int64]
        lib.oc_round_f16.restype = None
        lib.oc_round_f16.argtypes = [f32p, ctypes.c_int64]
        lib.oc_maxpool2d_nhwc.restype = ctypes.c_int
        lib.oc_maxpool2d_nhwc.argtypes = [f32p] + [ctypes.c_int] * 7 + [f32p]
        lib.oc_add_relu.restype = None
        lib.oc_add_relu.argtypes = [f32p, f32p, ctypes.c_int64, f32p]
        assert lib.oc_param_count() == 17
        _lib = lib
    return _lib


def _ptr(a: Optional[np.ndarray], ctype):
    if a is None:
        return ctypes.cast(None, ctypes.POINTER(ctype))
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _params(spec) -> np.ndarray:
    return np.array(
        [spec.n, spec.c_in, spec.h, spec.w, spec.c_out, spec.kh, spec.kw, spec.stride_h, spec.stride_w,
         spec.pad_h, spec.pad_w, spec.dil_h, spec.dil_w, 1 if spec.layout == "nchw" else 0,
         1 if spec.has_bias else 0, 1 if spec.relu else 0, 1 if spec.mask_mode == "spatial" else 0],
        dtype=np.int32,
    )


def num_threads() -> int:
    """OpenMP threads the oracle's loops run on."""
    return int(_load().oc_num_threads())


def out_size(inp: int, k: int, stride: int, pad: int, dil: int) -> int:
    return int(_load().oc_out_size(inp, k, stride, pad, dil))


def kept_count(sparsity: float, output_size: int) -> int:
    """Rows that stay in the contraction: output_size - sparsity*output_size (Sec. 3.2), half up."""
    return int(_load().oc_kept_count(float(sparsity), int(output_size)))


def compact_rows(mask: np.ndarray) -> np.ndarray:
    """Ascending list of the positions whose mask is 1 (Alg. 2, indirection init)."""
    mask = np.ascontiguousarray(mask, dtype=np.uint8).ravel()
    idx = np.empty(mask.size, dtype=np.int32)
    kept = _load().oc_compact_rows(_ptr(mask, ctypes.c_uint8), mask.size, _ptr(idx, ctypes.c_int32))
    if kept < 0:
        raise ValueError("mask bytes must be 0 or 1")
    return idx[:kept].copy()


def masked_conv2d(spec, x, w, bias, mask, want_absum: bool = False):
    """Dense-layout output of the masked convolution (float32, double accumulation).

    Returns ``y`` or ``(y, absum)``; ``absum`` is sum|x*w| + |bias| per output element.
    """
    lib = _load()
    x, w = _f32(x), _f32(w)
    assert x.shape == tuple(spec.x_shape()) and w.shape == tuple(spec.w_shape())
    mask = np.ascontiguousarray(mask, dtype=np.uint8).ravel()
    assert mask.size == spec.mask_len
    b = _f32(bias) if spec.has_bias else None
    if spec.has_bias:
        assert b.shape == (spec.c_out,)
    y = np.empty(spec.y_shape(), dtype=np.float32)
    absum = np.empty(spec.y_shape(), dtype=np.float64) if want_absum else None
    p = _params(spec)
    rc = lib.oc_masked_conv2d(_ptr(p, ctypes.c_int32), _ptr(x, ctypes.c_float), _ptr(w, ctypes.c_float),
                              _ptr(b, ctypes.c_float), _ptr(mask, ctypes.c_uint8), _ptr(y, ctypes.c_float),
                              _ptr(absum, ctypes.c_double))
    if rc != 0:
        raise ValueError(f"oracle rejected the problem (code {rc})")
    return (y, absum) if want_absum else y


def masked_conv2d_rows(spec, x, w, bias, mask, rows, want_absum: bool = False):
    """Output of selected rows r = (n*Ho + oy)*Wo + ox, shape [len(rows), Cout]."""
    lib = _load()
    x, w = _f32(x), _f32(w)
    assert x.shape == tuple(spec.x_shape()) and w.shape == tuple(spec.w_shape())
    mask = np.ascontiguousarray(mask, dtype=np.uint8).ravel()
    assert mask.size == spec.mask_len
    b = _f32(bias) if spec.has_bias else None
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    y = np.empty((rows.size, spec.c_out), dtype=np.float32)
    absum = np.empty((rows.size, spec.c_out), dtype=np.float64) if want_absum else None
    p = _params(spec)
    rc = lib.oc_masked_conv2d_rows(_ptr(p, ctypes.c_int32), _ptr(x, ctypes.c_float), _ptr(w, ctypes.c_float),
                                   _ptr(b, ctypes.c_float), _ptr(mask, ctypes.c_uint8), _ptr(rows, ctypes.c_int64),
                                   rows.size, _ptr(y, ctypes.c_float), _ptr(absum, ctypes.c_double))
    if rc != 0:
        raise ValueError(f"oracle rejected the problem (code {rc})")
    return (y, absum) if want_absum else y


def masked_conv2d_backward(spec, x, w, y, dy, mask, want_abs: bool = False):
    """Gradients of the masked convolution w.r.t. input, filters and bias (float64): ``(dx, dw, db)``, or
    ``(dx, dw, db, dx_abs, dw_abs)`` with the sums of absolute terms.  ``y`` is the forward output whose
    sign gates the ReLU; ``dy`` the upstream gradient (both in the output layout)."""
    lib = _load()
    x, w, y, dy = _f32(x), _f32(w), _f32(y), _f32(dy)
    assert x.shape == tuple(spec.x_shape()) and w.shape == tuple(spec.w_shape()) and spec.groups == 1
    assert y.shape == tuple(spec.y_shape()) and dy.shape == tuple(spec.y_shape())
    mask = np.ascontiguousarray(mask, dtype=np.uint8).ravel()
    assert mask.size == spec.mask_len
    dx, dw, db = np.empty(x.shape, np.float64), np.empty(w.shape, np.float64), np.empty(spec.c_out, np.float64)
    dxa = np.empty(x.shape, np.float64) if want_abs else None
    dwa = np.empty(w.shape, np.float64) if want_abs else None
    p = _params(spec)
    rc = lib.oc_masked_conv2d_backward(_ptr(p, ctypes.c_int32), _ptr(x, ctypes.c_float), _ptr(w, ctypes.c_float),
                                       _ptr(y, ctypes.c_float), _ptr(dy, ctypes.c_float), _ptr(mask, ctypes.c_uint8),
                                       _ptr(dx, ctypes.c_double), _ptr(dw, ctypes.c_double), _ptr(db, ctypes.c_double),
                                       _ptr(dxa, ctypes.c_double), _ptr(dwa, ctypes.c_double))
    if rc != 0:
        raise ValueError(f"oracle rejected the problem (code {rc})")
    return (dx, dw, db, dxa, dwa) if want_abs else (dx, dw, db)


def row_mask(spec, mask: np.ndarray) -> np.ndarray:
    """One mask byte per lowered row (a 2-D mask is shared by every image of the batch)."""
    mask = np.ascontiguousarray(mask, dtype=np.uint8).ravel()
    assert mask.size == spec.mask_len
    return mask if spec.mask_mode == "row" else np.tile(mask, spec.n)


def to_compact(t_dense: np.ndarray, mask_rows: np.ndarray) -> np.ndarray:
    """The kept rows of a dense NHWC map [N,H,W,C], ascending, as a matrix [kept, C]: what the GEMM
    of Sec. 3.2 stage (ii) leaves before the zeros are re-inserted."""
    m = mask_rows.size
    c = t_dense.size // m
    return np.ascontiguousarray(t_dense.reshape(m, c)[mask_rows == 1])


def from_compact(t_compact: np.ndarray, mask_rows: np.ndarray, shape) -> np.ndarray:
    """Alg. 2 post-processing: the compact rows placed at their dense positions, +0.0 elsewhere."""
    m = mask_rows.size
    t_compact = np.asarray(t_compact)
    out = np.zeros((m, t_compact.shape[1]), dtype=t_compact.dtype)
    out[mask_rows == 1] = t_compact
    return out.reshape(shape)


def masked_conv2d_compact(spec, x, w, bias, mask, x_compact: bool = False, y_compact: bool = False):
    """The masked convolution with compact operands (NHWC only).

    x_compact: ``x`` is [kept, Cin], the kept rows of the layer's input map -- only a 1x1 stride-1
    unpadded layer can take it (its window is the pixel itself, so the dropped pixels of the input are
    never read by a kept output row).  y_compact: the result is [kept, Cout] instead of the dense map.
    Both are defined through the dense-layout convolution: expand, convolve, take the kept rows.
    """
    assert spec.layout == "nhwc"
    rm = row_mask(spec, mask)
    if x_compact:
        assert (spec.kh, spec.kw, spec.stride_h, spec.stride_w, spec.pad_h, spec.pad_w) == (1, 1, 1, 1, 0, 0)
        x = from_compact(_f32(x), rm, spec.x_shape())
    y = masked_conv2d(spec, x, w, bias, mask)
    return to_compact(y, rm) if y_compact else y


def masked_conv2d_residual(spec, x, w, bias, mask, residual, post_relu: bool, x_compact: bool = False,
                           y_compact: bool = False):
    """The masked convolution followed by a shortcut sum, as one operator:

        y = post( masked_conv2d(x) + residual ),   post = ReLU or identity

    i.e. what a block computes when the sum (ResNet: ReLU after it; inverted-residual blocks: linear) follows the
    layer directly.  A dropped row of the convolution is +0.0 (Alg. 2), so there y = post(residual): the sum is not
    masked.  ``residual`` has the format of the result (dense map, or [kept, Cout] when y_compact).  Defined through
    the dense-layout operators in double precision; the layer's own activation (spec.relu) acts before the sum."""
    if x_compact or y_compact:
        conv = masked_conv2d_compact(spec, x, w, bias, mask, x_compact=x_compact, y_compact=y_compact)
    else:
        conv = masked_conv2d(spec, x, w, bias, mask)      # (any layout)
    res = _f32(residual)
    assert res.shape == conv.shape or res.size == conv.size
    y = conv.astype(np.float64) + res.reshape(conv.shape).astype(np.float64)
    if post_relu:
        y = np.maximum(y, 0.0)
    return y.astype(np.float32)


def masked_depthwise_conv2d(spec, x, w, bias, mask, want_absum: bool = False):
    """Masked depthwise convolution (groups == Cin == Cout, NHWC): channel c of the output is the
    kh x kw cross-correlation of channel c of the input with filter w[c, :, :, 0]; the mask removes output
    pixels exactly as in Sec. 3 (a dropped pixel is +0.0 in every channel, no bias, no activation).

    The paper speaks of convolutional layers in general and times networks with depthwise layers; it
    does not spell out this case -- the reading is the masking semantics of Sec. 3 applied unchanged.
    Direct loop nest over output pixels and taps, double accumulation.
    """
    assert spec.layout == "nhwc" and spec.groups == spec.c_in == spec.c_out
    x64 = np.asarray(x, dtype=np.float32).astype(np.float64)
    w64 = np.asarray(w, dtype=np.float32).astype(np.float64).reshape(spec.c_out, spec.kh, spec.kw)
    assert x64.shape == tuple(spec.x_shape())
    b64 = np.asarray(bias, dtype=np.float32).astype(np.float64) if spec.has_bias else None
    rm = row_mask(spec, mask).reshape(spec.n, spec.ho, spec.wo)
    y = np.zeros(spec.y_shape(), dtype=np.float64)
    absum = np.zeros(spec.y_shape(), dtype=np.float64)
    for oy in range(spec.ho):
        for ox in range(spec.wo):
            acc = np.zeros((spec.n, spec.c_out), dtype=np.float64)
            mag = np.zeros((spec.n, spec.c_out), dtype=np.float64)
            for ky in range(spec.kh):
                iy = oy * spec.stride_h - spec.pad_h + ky * spec.dil_h
                if iy < 0 or iy >= spec.h:
                    continue
                for kx in range(spec.kw):
                    ix = ox * spec.stride_w - spec.pad_w + kx * spec.dil_w
                    if ix < 0 or ix >= spec.w:
                        continue
                    term = x64[:, iy, ix, :] * w64[None, :, ky, kx]
                    acc = acc + term
                    mag = mag + np.abs(term)
            if b64 is not None:
                acc = acc + b64[None, :]
                mag = mag + np.abs(b64)[None, :]
            if spec.relu:
                acc = np.maximum(acc, 0.0)
            keep = rm[:, oy, ox][:, None] == 1
            y[:, oy, ox, :] = np.where(keep, acc, 0.0)
            absum[:, oy, ox, :] = np.where(keep, mag, 0.0)
    y = y.astype(np.float32)
    return (y, absum) if want_absum else y


def masked_depthwise_conv2d_compact(spec, x, w, bias, mask, x_mask=None, y_compact: bool = False):
    """The masked depthwise convolution with compact operands (NHWC).

    x_mask: when given, ``x`` is [kept_in, C] -- the rows that ``x_mask`` keeps of the layer's input map (one
    byte per input pixel and image in row mode, one per input pixel in spatial mode: the mask of the layer
    that produced the map).  The dropped input pixels are +0.0, which is what Alg. 2 writes there, so unlike
    a 1x1 layer a window may read them.  y_compact: the result is [kept, C] instead of the dense map.
    Both are defined through the dense-layout convolution: expand, convolve, take the kept rows."""
    assert spec.layout == "nhwc"
    if x_mask is not None:
        xm = np.ascontiguousarray(x_mask, dtype=np.uint8).ravel()
        pixels = spec.h * spec.w
        assert xm.size == (spec.n * pixels if spec.mask_mode == "row" else pixels)
        in_rows = xm if spec.mask_mode == "row" else np.tile(xm, spec.n)
        x = from_compact(_f32(x), in_rows, spec.x_shape())
    y = masked_depthwise_conv2d(spec, x, w, bias, mask)
    return to_compact(y, row_mask(spec, mask)) if y_compact else y


def round_storage(a: np.ndarray, dtype: str) -> np.ndarray:
    """Round float32 values to the storage type of a layer output (nearest even), widened back."""
    a = np.array(a, dtype=np.float32, order="C", copy=True)
    if dtype == "bf16":
        _load().oc_round_bf16(_ptr(a, ctypes.c_float), a.size)
    elif dtype == "f16":
        _load().oc_round_f16(_ptr(a, ctypes.c_float), a.size)
    elif dtype != "f32":
        raise ValueError(dtype)
    return a


def maxpool2d_nhwc(x: np.ndarray, k: int = 3, s: int = 2, p: int = 1) -> np.ndarray:
    x = _f32(x)
    n, h, w, c = x.shape
    ho, wo = out_size(h, k, s, p, 1), out_size(w, k, s, p, 1)
    y = np.empty((n, ho, wo, c), dtype=np.float32)
    rc = _load().oc_maxpool2d_nhwc(_ptr(x, ctypes.c_float), n, h, w, c, k, s, p, _ptr(y, ctypes.c_float))
    if rc != 0:
        raise ValueError("bad pooling geometry")
    return y


def add_relu(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    a, b = _f32(a), _f32(b)
    assert a.shape == b.shape
    y = np.empty_like(a)
    _load().oc_add_relu(_ptr(a, ctypes.c_float), _ptr(b, ctypes.c_float), a.size, _ptr(y, ctypes.c_float))
    return y


def run_network(ops, tensors: Dict[str, np.ndarray], layer_inputs, absums: Optional[Dict[str, np.ndarray]] = None
                ) -> Dict[str, np.ndarray]:
    """Interpret a list of workload ops on the CPU.

    ``tensors`` holds the named inputs (float32, values representable in the storage dtype);
    ``layer_inputs(spec)`` returns (w, bias, mask) for a conv.  Every op's result is rounded to
    the storage dtype, as a runtime that keeps activations in that dtype would.
    ``absums``: when a dict is passed it receives, per convolution output, the sum of the magnitudes of
    every product and the bias behind each element (the condition-aware error bound of the layer tests).
    """
    t = dict(tensors)
    for op in ops:
        if op.kind == "conv":
            w, b, m = layer_inputs(op.spec)
            conv = masked_depthwise_conv2d if op.spec.groups > 1 else masked_conv2d
            if absums is not None:
                y, absums[op.out] = conv(op.spec, t[op.src], w, b, m, want_absum=True)
            else:
                y = conv(op.spec, t[op.src], w, b, m)
            t[op.out] = round_storage(y, op.spec.dtype)
        elif op.kind == "maxpool":
            t[op.out] = maxpool2d_nhwc(t[op.src], 3, 2, 1)
        elif op.kind == "add_relu":
            dt = next(o.spec.dtype for o in ops if o.kind == "conv")
            t[op.out] = round_storage(add_relu(t[op.src], t[op.src2]), dt)
        elif op.kind == "add":
            dt = next(o.spec.dtype for o in ops if o.kind == "conv")
            t[op.out] = round_storage((_f32(t[op.src]).astype(np.float64) + _f32(t[op.src2])).astype(np.float32), dt)
        else:
            raise ValueError(op.kind)
    return t
