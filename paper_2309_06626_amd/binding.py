"""ctypes binding of libsparse_conv.so: argument marshalling only.

Every function has the name and meaning of its C entry point (include/sparse_conv.h).  PyTorch
supplies device memory (tensors) and the stream handle; all arithmetic runs in the HIP kernels.
There is no CPU fallback: if the library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch  # must be imported before the library so both share one HIP runtime

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsparse_conv.so")

SC_OK = 0
SC_ERR_NULL, SC_ERR_BAD_SHAPE, SC_ERR_UNSUPPORTED, SC_ERR_MASK_COUNT = 1, 2, 3, 4
SC_ERR_WORKSPACE, SC_ERR_ALIGN, SC_ERR_HIP = 5, 6, 7
SC_F32, SC_F16, SC_BF16 = 0, 1, 2
SC_NHWC, SC_NCHW = 0, 1
SC_MASK_ROW, SC_MASK_SPATIAL = 0, 1
SC_OUT_ZERO_FILL, SC_OUT_SCATTER_ONLY = 0, 1

DTYPE_CODE = {"f32": SC_F32, "f16": SC_F16, "bf16": SC_BF16}
TORCH_DTYPE = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}
_CODE_OF_TORCH = {torch.float32: SC_F32, torch.float16: SC_F16, torch.bfloat16: SC_BF16}


class sc_conv_desc(ctypes.Structure):
    _fields_ = [(name, ctypes.c_int32) for name in (
        "n", "c_in", "h", "w", "c_out", "kh", "kw", "stride_h", "stride_w", "pad_h", "pad_w", "dil_h", "dil_w",
        "groups", "dtype", "layout", "has_bias", "relu", "mask_mode", "out_mode")] + [("sparsity", ctypes.c_float)]


class ScError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().sc_status_string(status).decode()
        if status == SC_ERR_HIP:
            msg += f" [hipError {lib().sc_last_hip_error()}]"
        super().__init__(f"{where}: {msg}")


_lib = None


def lib() -> ctypes.CDLL:
    """Load the shared library (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2309_06626_amd.build` "
                "(there is no fallback implementation)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
        pd = ctypes.POINTER(sc_conv_desc)
        L.sparse_conv_output_shape.restype = ctypes.c_int
        L.sparse_conv_output_shape.argtypes = [pd, ctypes.POINTER(i32), ctypes.POINTER(i32), ctypes.POINTER(i64)]
        L.sparse_conv_workspace_bytes.restype = ctypes.c_int
        L.sparse_conv_workspace_bytes.argtypes = [pd, ctypes.POINTER(ctypes.c_size_t)]
        L.sparse_conv_plan.restype = ctypes.c_int
        L.sparse_conv_plan.argtypes = [pd, vp, vp, vp, ctypes.c_size_t, vp, ctypes.POINTER(vp)]
        L.sparse_conv_plan_set_mask.restype = ctypes.c_int
        L.sparse_conv_plan_set_mask.argtypes = [vp, vp, vp]
        L.sparse_conv_plan_set_filters.restype = ctypes.c_int
        L.sparse_conv_plan_set_filters.argtypes = [vp, vp, vp]
        L.sparse_conv_run.restype = ctypes.c_int
        L.sparse_conv_run.argtypes = [vp, vp, vp, vp, vp]
        L.sparse_conv_run_rows.restype = ctypes.c_int
        L.sparse_conv_run_rows.argtypes = [vp, vp, i32, vp, vp, i32, vp]
        L.dense_conv_run.restype = ctypes.c_int
        L.dense_conv_run.argtypes = [vp, vp, vp, vp, vp]
        L.sparse_conv_plan_info.restype = ctypes.c_int
        L.sparse_conv_plan_info.argtypes = [vp, ctypes.POINTER(i64), ctypes.POINTER(i64), ctypes.POINTER(i32),
                                            ctypes.POINTER(i32), ctypes.POINTER(vp)]
        L.sparse_conv_plan_tiles.restype = ctypes.c_int
        L.sparse_conv_plan_tiles.argtypes = [vp, i32, ctypes.POINTER(i32), ctypes.POINTER(i32), ctypes.POINTER(i64)]
        L.sparse_conv_plan_kernel.restype = ctypes.c_char_p
        L.sparse_conv_plan_kernel.argtypes = [vp, i32]
        L.sparse_conv_plan_fused_kernel.restype = ctypes.c_char_p
        L.sparse_conv_plan_fused_kernel.argtypes = [vp, i32]
        L.sparse_conv_plan_set_tiles.restype = ctypes.c_int
        L.sparse_conv_plan_set_tiles.argtypes = [vp, i32, i32, i32]
        L.sparse_conv_plan_set_option.restype = ctypes.c_int
        L.sparse_conv_plan_set_option.argtypes = [vp, i32, i32]
        L.sparse_conv_plan_destroy.restype = None
        L.sparse_conv_plan_destroy.argtypes = [vp]
        L.sc_status_string.restype = ctypes.c_char_p
        L.sc_status_string.argtypes = [ctypes.c_int]
        L.sc_last_hip_error.restype = i32
        L.sc_last_hip_error.argtypes = []
        L.sc_maxpool2d_nhwc.restype = ctypes.c_int
        L.sc_maxpool2d_nhwc.argtypes = [vp, vp] + [i32] * 8 + [vp]
        L.sc_add_relu.restype = ctypes.c_int
        L.sc_add_relu.argtypes = [vp, vp, vp, i32, i64, vp]
        L.sparse_conv_plan_set_input_mask.restype = ctypes.c_int
        L.sparse_conv_plan_set_input_mask.argtypes = [vp, vp, ctypes.POINTER(i64), vp]
        L.sparse_conv_run_residual.restype = ctypes.c_int
        L.sparse_conv_run_residual.argtypes = [vp, vp, i32, vp, vp, i32, vp, i32, vp]
        L.dense_conv_run_residual.restype = ctypes.c_int
        L.dense_conv_run_residual.argtypes = [vp, vp, vp, vp, i32, vp, vp]
        L.sc_add.restype = ctypes.c_int
        L.sc_add.argtypes = [vp, vp, vp, i32, i64, vp]
        L.sparse_conv_plan_mask.restype = vp
        L.sparse_conv_plan_mask.argtypes = [vp]
        L.sparse_conv_backward_workspace_bytes.restype = ctypes.c_int
        L.sparse_conv_backward_workspace_bytes.argtypes = [pd, ctypes.POINTER(ctypes.c_size_t)]
        L.sparse_conv_backward_plan.restype = ctypes.c_int
        L.sparse_conv_backward_plan.argtypes = [vp, pd, vp, vp, ctypes.c_size_t, vp, ctypes.POINTER(vp)]
        L.sparse_conv_backward_set_filters.restype = ctypes.c_int
        L.sparse_conv_backward_set_filters.argtypes = [vp, vp, vp]
        L.sparse_conv_backward_run.restype = ctypes.c_int
        L.sparse_conv_backward_run.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp]
        L.sparse_conv_backward_destroy.restype = None
        L.sparse_conv_backward_destroy.argtypes = [vp]
        L.sparse_conv_plan_tune.restype = ctypes.c_int
        L.sparse_conv_plan_tune.argtypes = [vp, vp, vp, vp, vp]
        L.sc_probe_stream_copy.restype = ctypes.c_int
        L.sc_probe_stream_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
        L.sc_probe_mfma_bf16.restype = ctypes.c_int
        L.sc_probe_mfma_bf16.argtypes = [i32, i32, vp, ctypes.POINTER(ctypes.c_double), vp]
        L.sparse_mask_workspace_bytes.restype = ctypes.c_int
        L.sparse_mask_workspace_bytes.argtypes = [i32, i32, ctypes.POINTER(ctypes.c_size_t)]
        L.sparse_mask_generate.restype = ctypes.c_int
        L.sparse_mask_generate.argtypes = [vp, i32, i32, i32, i32, ctypes.c_float, vp, vp, ctypes.c_size_t, vp]
        L.sparse_mask_generate_static.restype = ctypes.c_int
        L.sparse_mask_generate_static.argtypes = [vp, i32, i32, i32, i32, ctypes.c_float, vp, vp]
        _lib = L
    return _lib


def make_desc(n, c_in, h, w, c_out, kh=3, kw=3, stride_h=1, stride_w=1, pad_h=1, pad_w=1, dil_h=1, dil_w=1,
              groups=1, dtype=SC_BF16, layout=SC_NHWC, has_bias=1, relu=1, mask_mode=SC_MASK_ROW,
              out_mode=SC_OUT_ZERO_FILL, sparsity=-1.0) -> sc_conv_desc:
    return sc_conv_desc(n, c_in, h, w, c_out, kh, kw, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w, groups,
                        dtype, layout, int(has_bias), int(relu), mask_mode, out_mode, float(sparsity))


def desc_from_spec(spec, out_mode=SC_OUT_ZERO_FILL, check_count=True) -> sc_conv_desc:
    """Descriptor of a workloads.ConvSpec."""
    return make_desc(spec.n, spec.c_in, spec.h, spec.w, spec.c_out, spec.kh, spec.kw, spec.stride_h, spec.stride_w,
                     spec.pad_h, spec.pad_w, spec.dil_h, spec.dil_w, getattr(spec, "groups", 1), DTYPE_CODE[spec.dtype],
                     SC_NCHW if spec.layout == "nchw" else SC_NHWC, spec.has_bias, spec.relu,
                     SC_MASK_SPATIAL if spec.mask_mode == "spatial" else SC_MASK_ROW, out_mode,
                     spec.sparsity if check_count else -1.0)


def _check(status: int, where: str):
    if status != SC_OK:
        raise ScError(status, where)


def _stream_handle(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream) if hasattr(stream, "cuda_stream") else int(stream)


def _dev_ptr(t: Optional[torch.Tensor], what: str) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{what} must be a device tensor")
    if not t.is_contiguous():
        raise ValueError(f"{what} must be contiguous")
    return t.data_ptr()


def sparse_conv_output_shape(desc: sc_conv_desc) -> Tuple[int, int, int]:
    ho, wo, m = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int64()
    _check(lib().sparse_conv_output_shape(ctypes.byref(desc), ctypes.byref(ho), ctypes.byref(wo), ctypes.byref(m)),
           "sparse_conv_output_shape")
    return ho.value, wo.value, m.value


def sparse_conv_workspace_bytes(desc: sc_conv_desc) -> int:
    n = ctypes.c_size_t()
    _check(lib().sparse_conv_workspace_bytes(ctypes.byref(desc), ctypes.byref(n)), "sparse_conv_workspace_bytes")
    return n.value


class Plan:
    """Owner of an sc_plan handle and of the tensors the plan points into."""

    def __init__(self, handle: int, desc: sc_conv_desc, workspace: torch.Tensor):
        self.handle = handle
        self.desc = desc
        self.workspace = workspace  # keeps the device memory alive
        self.x_kept = None          # rows of a compact input after sparse_conv_plan_set_input_mask

    def close(self):
        if self.handle:
            lib().sparse_conv_plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def sparse_conv_plan(desc: sc_conv_desc, mask: torch.Tensor, w: torch.Tensor,
                     workspace: Optional[torch.Tensor] = None, stream=None) -> Plan:
    """mask: uint8 device tensor; w: filters in the descriptor's layout/dtype (device)."""
    if mask.dtype != torch.uint8:
        raise ValueError("mask must be uint8")
    if _CODE_OF_TORCH.get(w.dtype) != desc.dtype:
        raise ValueError("filter dtype does not match the descriptor")
    nbytes = sparse_conv_workspace_bytes(desc)    # also validates the descriptor
    ho, wo, m = sparse_conv_output_shape(desc)
    want_mask = m if desc.mask_mode == SC_MASK_ROW else ho * wo
    want_w = desc.c_out * desc.kh * desc.kw * (desc.c_in // desc.groups)
    if mask.numel() != want_mask:
        raise ValueError(f"mask holds {mask.numel()} bytes, the layer needs {want_mask}")
    if w.numel() != want_w:
        raise ValueError(f"filters hold {w.numel()} elements, the layer needs {want_w}")
    if workspace is None:
        workspace = torch.empty(nbytes, dtype=torch.uint8, device=mask.device)
    out = ctypes.c_void_p()
    st = lib().sparse_conv_plan(ctypes.byref(desc), _dev_ptr(mask, "mask"), _dev_ptr(w, "w"),
                                _dev_ptr(workspace, "workspace"), workspace.numel(), _stream_handle(stream),
                                ctypes.byref(out))
    _check(st, "sparse_conv_plan")
    return Plan(out.value, desc, workspace)


def _check_operands(plan: Plan, x, bias, y, x_compact=False, y_compact=False):
    """The library cannot see tensor sizes: a wrong one would be an out-of-bounds access on the GPU."""
    d = plan.desc
    for t, what in ((x, "x"), (y, "y")):
        if _CODE_OF_TORCH.get(t.dtype) != d.dtype:
            raise ValueError(f"{what} dtype does not match the plan")
    if bias is not None and (bias.dtype != torch.float32 or bias.numel() != d.c_out):
        raise ValueError("bias must be float32[c_out]")
    info = sparse_conv_plan_info(plan)
    # a compact input holds this layer's kept pixels (1x1 windows) or, for a depthwise layer with windows, the
    # pixels its input mask keeps (sparse_conv_plan_set_input_mask)
    x_rows = getattr(plan, "x_kept", None) if (d.groups > 1 and d.kh * d.kw > 1) else info["kept"]
    if x_compact and x_rows is None:
        raise ValueError("a compact input of this layer needs sparse_conv_plan_set_input_mask first")
    want_x = x_rows * d.c_in if x_compact else d.n * d.h * d.w * d.c_in
    want_y = (info["kept"] if y_compact else info["m"]) * d.c_out
    if x.numel() != want_x:
        raise ValueError(f"x holds {x.numel()} elements, the plan needs {want_x}")
    if y.numel() != want_y:
        raise ValueError(f"y holds {y.numel()} elements, the plan needs {want_y}")


def sparse_conv_plan_set_mask(plan: Plan, mask: torch.Tensor, stream=None):
    """A new mask for an existing plan (re-runs the compaction; synchronises the stream)."""
    d = plan.desc
    info = sparse_conv_plan_info(plan)
    want = info["m"] if d.mask_mode == SC_MASK_ROW else info["ho"] * info["wo"]
    if mask.dtype != torch.uint8 or mask.numel() != want:
        raise ValueError(f"mask must hold {want} bytes")
    _check(lib().sparse_conv_plan_set_mask(plan.handle, _dev_ptr(mask, "mask"), _stream_handle(stream)),
           "sparse_conv_plan_set_mask")


def sparse_conv_plan_set_filters(plan: Plan, w: torch.Tensor, stream=None):
    """New filter values for an existing plan (same layout and dtype)."""
    d = plan.desc
    if _CODE_OF_TORCH.get(w.dtype) != d.dtype or w.numel() != d.c_out * d.kh * d.kw * (d.c_in // d.groups):
        raise ValueError("filters do not match the plan")
    _check(lib().sparse_conv_plan_set_filters(plan.handle, _dev_ptr(w, "w"), _stream_handle(stream)),
           "sparse_conv_plan_set_filters")


def _run(fn, name, plan: Plan, x, bias, y, stream):
    _check_operands(plan, x, bias, y)
    _check(fn(plan.handle, _dev_ptr(x, "x"), _dev_ptr(bias, "bias"), _dev_ptr(y, "y"), _stream_handle(stream)), name)
    return y


def sparse_conv_run(plan: Plan, x: torch.Tensor, bias: Optional[torch.Tensor], y: torch.Tensor, stream=None):
    return _run(lib().sparse_conv_run, "sparse_conv_run", plan, x, bias, y, stream)


SC_ROWS_DENSE, SC_ROWS_COMPACT = 0, 1


def sparse_conv_run_rows(plan: Plan, x: torch.Tensor, bias: Optional[torch.Tensor], y: torch.Tensor,
                         x_rows: int = SC_ROWS_DENSE, y_rows: int = SC_ROWS_DENSE, stream=None):
    """sparse_conv_run with compact operands: x = [kept, Cin] and / or y = [kept, Cout]."""
    _check_operands(plan, x, bias, y, x_rows == SC_ROWS_COMPACT, y_rows == SC_ROWS_COMPACT)
    _check(lib().sparse_conv_run_rows(plan.handle, _dev_ptr(x, "x"), x_rows, _dev_ptr(bias, "bias"), _dev_ptr(y, "y"),
                                      y_rows, _stream_handle(stream)), "sparse_conv_run_rows")
    return y


def prepared_run_rows(plan: Plan, x: torch.Tensor, bias: Optional[torch.Tensor], y: torch.Tensor,
                      x_rows: int = SC_ROWS_DENSE, y_rows: int = SC_ROWS_DENSE, stream=None):
    """Like prepared_run, for sparse_conv_run_rows."""
    sparse_conv_run_rows(plan, x, bias, y, x_rows, y_rows, stream)
    fn, h, px, pb, py, st = lib().sparse_conv_run_rows, plan.handle, x.data_ptr(), \
        (bias.data_ptr() if bias is not None else None), y.data_ptr(), _stream_handle(stream)
    keep = (plan, x, bias, y)

    def call(stream_handle=None):
        rc = fn(h, px, x_rows, pb, py, y_rows, st if stream_handle is None else stream_handle)
        if rc != SC_OK:
            raise ScError(rc, "sparse_conv_run_rows")
        return keep[3]

    return call


def _check_residual(residual: torch.Tensor, y: torch.Tensor):
    if residual.dtype != y.dtype or residual.numel() != y.numel():
        raise ValueError("the shortcut tensor must have the dtype and size of y")
    if residual.data_ptr() == y.data_ptr():
        raise ValueError("the shortcut tensor must not overlap y")


def sparse_conv_run_residual(plan: Plan, x: torch.Tensor, bias: Optional[torch.Tensor], residual: torch.Tensor,
                             y: torch.Tensor, residual_relu: bool = False, x_rows: int = SC_ROWS_DENSE,
                             y_rows: int = SC_ROWS_DENSE, dense: bool = False, stream=None):
    """y = post(act(conv + bias) + residual): sparse_conv_run_residual, or dense_conv_run_residual with dense=True."""
    return prepared_run_residual(plan, x, bias, residual, y, residual_relu, x_rows, y_rows, dense, stream)()


def prepared_run_residual(plan: Plan, x: torch.Tensor, bias: Optional[torch.Tensor], residual: torch.Tensor,
                          y: torch.Tensor, residual_relu: bool = False, x_rows: int = SC_ROWS_DENSE,
                          y_rows: int = SC_ROWS_DENSE, dense: bool = False, stream=None):
    """Validated once; the returned callable issues the fused run (no launch happens here)."""
    if dense and (x_rows != SC_ROWS_DENSE or y_rows != SC_ROWS_DENSE):
        raise ValueError("a dense run has dense operands")
    _check_operands(plan, x, bias, y, x_rows == SC_ROWS_COMPACT, y_rows == SC_ROWS_COMPACT)
    _check_residual(residual, y)
    L = lib()
    h, px, pb, pr, py, st = plan.handle, _dev_ptr(x, "x"), _dev_ptr(bias, "bias"), _dev_ptr(residual, "residual"), \
        _dev_ptr(y, "y"), _stream_handle(stream)
    rr = 1 if residual_relu else 0
    keep = (plan, x, bias, residual, y)

    def call(stream_handle=None):
        s = st if stream_handle is None else stream_handle
        if dense:
            rc = L.dense_conv_run_residual(h, px, pb, pr, rr, py, s)
        else:
            rc = L.sparse_conv_run_residual(h, px, x_rows, pb, pr, rr, py, y_rows, s)
        if rc != SC_OK:
            raise ScError(rc, "dense_conv_run_residual" if dense else "sparse_conv_run_residual")
        return keep[4]

    return call


def sparse_conv_plan_tune(plan: Plan, x: torch.Tensor, bias: Optional[torch.Tensor], y: torch.Tensor, stream=None):
    """Times the plan's candidate launches on these buffers and keeps the fastest (y ends up holding the sparse run)."""
    return _run(lib().sparse_conv_plan_tune, "sparse_conv_plan_tune", plan, x, bias, y, stream)


def dense_conv_run(plan: Plan, x: torch.Tensor, bias: Optional[torch.Tensor], y: torch.Tensor, stream=None):
    return _run(lib().dense_conv_run, "dense_conv_run", plan, x, bias, y, stream)


def prepared_run(plan: Plan, x: torch.Tensor, bias: Optional[torch.Tensor], y: torch.Tensor, dense: bool = False,
                 stream=None):
    """Validate once and return a zero-argument callable that issues the same run again
    (launch loops: the per-call marshalling cost of `_run` is paid once)."""
    fn = lib().dense_conv_run if dense else lib().sparse_conv_run
    name = "dense_conv_run" if dense else "sparse_conv_run"
    _run(fn, name, plan, x, bias, y, stream)   # full checks, one real launch
    h, px, pb, py, st = plan.handle, x.data_ptr(), (bias.data_ptr() if bias is not None else None), y.data_ptr(), \
        _stream_handle(stream)
    keep = (plan, x, bias, y)

    def call(stream_handle=None):
        rc = fn(h, px, pb, py, st if stream_handle is None else stream_handle)
        if rc != SC_OK:
            raise ScError(rc, name)
        return keep[3]

    return call


def sparse_conv_plan_info(plan: Plan) -> dict:
    m, kept, ho, wo, rows = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int32(), ctypes.c_int32(), ctypes.c_void_p()
    _check(lib().sparse_conv_plan_info(plan.handle, ctypes.byref(m), ctypes.byref(kept), ctypes.byref(ho),
                                       ctypes.byref(wo), ctypes.byref(rows)), "sparse_conv_plan_info")
    return {"m": m.value, "kept": kept.value, "ho": ho.value, "wo": wo.value, "row_idx_ptr": rows.value}


def plan_row_idx(plan: Plan) -> torch.Tensor:
    """Copy of the kept-row list (int32, ascending) as a device tensor."""
    info = sparse_conv_plan_info(plan)
    off = info["row_idx_ptr"] - plan.workspace.data_ptr()
    return plan.workspace[off: off + 4 * info["kept"]].view(torch.int32).clone()


def sparse_conv_plan_tiles(plan: Plan, which: int) -> Tuple[int, int, int]:
    tm, tn, wg = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int64()
    _check(lib().sparse_conv_plan_tiles(plan.handle, which, ctypes.byref(tm), ctypes.byref(tn), ctypes.byref(wg)),
           "sparse_conv_plan_tiles")
    return tm.value, tn.value, wg.value


def sparse_conv_plan_kernel(plan: Plan, which: int) -> str:
    name = lib().sparse_conv_plan_kernel(plan.handle, which)
    if name is None:
        raise ScError(SC_ERR_UNSUPPORTED, "sparse_conv_plan_kernel (bad plan or launch selector)")
    return name.decode()


def sparse_conv_plan_fused_kernel(plan: Plan, which: int) -> str:
    name = lib().sparse_conv_plan_fused_kernel(plan.handle, which)
    if name is None:
        raise ScError(SC_ERR_UNSUPPORTED, "sparse_conv_plan_fused_kernel (bad launch selector, or a plan without a fused form)")
    return name.decode()


def sparse_conv_plan_set_tiles(plan: Plan, which: int, tile_m: int, tile_n: int):
    _check(lib().sparse_conv_plan_set_tiles(plan.handle, which, tile_m, tile_n), "sparse_conv_plan_set_tiles")


SC_OPT_GATHER_PIPELINE = 0
SC_OPT_SPLIT_K = 1
SC_OPT_ROW_PANEL = 2
SC_OPT_STREAM_K = 3
SC_OPT_MASKED_STORE = 4
SC_OPT_SLAB = 5


def sparse_conv_plan_set_option(plan: Plan, option: int, value: int):
    _check(lib().sparse_conv_plan_set_option(plan.handle, option, value), "sparse_conv_plan_set_option")


def sc_maxpool2d_nhwc(x: torch.Tensor, k: int = 3, s: int = 2, p: int = 1, stream=None) -> torch.Tensor:
    n, h, w, c = x.shape
    ho, wo = (h + 2 * p - k) // s + 1, (w + 2 * p - k) // s + 1
    y = torch.empty((n, ho, wo, c), dtype=x.dtype, device=x.device)
    _check(lib().sc_maxpool2d_nhwc(_dev_ptr(x, "x"), _dev_ptr(y, "y"), _CODE_OF_TORCH[x.dtype], n, h, w, c, k, s, p,
                                   _stream_handle(stream)), "sc_maxpool2d_nhwc")
    return y


def prepared_maxpool(x: torch.Tensor, y: torch.Tensor, k: int = 3, s: int = 2, p: int = 1, stream=None):
    """Like prepared_run, for sc_maxpool2d_nhwc into a caller-owned output."""
    n, h, w, c = x.shape
    ho, wo = (h + 2 * p - k) // s + 1, (w + 2 * p - k) // s + 1
    if tuple(y.shape) != (n, ho, wo, c) or y.dtype != x.dtype:
        raise ValueError("output tensor does not match the pooled shape")
    fn, px, py, code, st = lib().sc_maxpool2d_nhwc, _dev_ptr(x, "x"), _dev_ptr(y, "y"), _CODE_OF_TORCH[x.dtype], \
        _stream_handle(stream)
    keep = (x, y)

    def call(stream_handle=None):
        _check(fn(px, py, code, n, h, w, c, k, s, p, st if stream_handle is None else stream_handle), "sc_maxpool2d_nhwc")
        return keep[1]

    call()
    return call


def sparse_conv_plan_set_input_mask(plan: "Plan", mask_in: torch.Tensor, stream=None) -> int:
    """Row list of a compact input of a depthwise layer with windows; returns the rows x must hold."""
    d = plan.desc
    want = d.h * d.w * (d.n if d.mask_mode == SC_MASK_ROW else 1)
    if mask_in.dtype != torch.uint8 or mask_in.numel() != want:
        raise ValueError(f"input mask must be uint8 with {want} entries")
    kept = ctypes.c_int64()
    _check(lib().sparse_conv_plan_set_input_mask(plan.handle, _dev_ptr(mask_in, "mask_in"), ctypes.byref(kept),
                                                 _stream_handle(stream)), "sparse_conv_plan_set_input_mask")
    plan.x_kept = int(kept.value)
    return plan.x_kept


def prepared_add(a: torch.Tensor, b: torch.Tensor, y: torch.Tensor, relu: bool = False, stream=None):
    """Like prepared_run, for sc_add (relu=False) or sc_add_relu into a caller-owned output."""
    if a.shape != b.shape or a.dtype != b.dtype or y.shape != a.shape or y.dtype != a.dtype:
        raise ValueError("operands differ in shape or dtype")
    name = "sc_add_relu" if relu else "sc_add"
    fn, pa, pb, py, code, n, st = getattr(lib(), name), _dev_ptr(a, "a"), _dev_ptr(b, "b"), _dev_ptr(y, "y"), \
        _CODE_OF_TORCH[a.dtype], a.numel(), _stream_handle(stream)
    keep = (a, b, y)

    def call(stream_handle=None):
        _check(fn(pa, pb, py, code, n, st if stream_handle is None else stream_handle), name)
        return keep[2]

    call()
    return call


def prepared_add_relu(a: torch.Tensor, b: torch.Tensor, y: torch.Tensor, stream=None):
    return prepared_add(a, b, y, relu=True, stream=stream)


def _add(name: str, a: torch.Tensor, b: torch.Tensor, y: Optional[torch.Tensor], stream) -> torch.Tensor:
    if a.shape != b.shape or a.dtype != b.dtype:
        raise ValueError("operands differ in shape or dtype")
    if y is None:
        y = torch.empty_like(a)
    elif y.shape != a.shape or y.dtype != a.dtype:
        raise ValueError("output differs from the operands in shape or dtype")
    _check(getattr(lib(), name)(_dev_ptr(a, "a"), _dev_ptr(b, "b"), _dev_ptr(y, "y"), _CODE_OF_TORCH[a.dtype],
                                a.numel(), _stream_handle(stream)), name)
    return y


def sc_add_relu(a: torch.Tensor, b: torch.Tensor, y: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    return _add("sc_add_relu", a, b, y, stream)


def sc_add(a: torch.Tensor, b: torch.Tensor, y: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    return _add("sc_add", a, b, y, stream)


def sparse_mask_workspace_bytes(ho: int, wo: int) -> int:
    out = ctypes.c_size_t()
    _check(lib().sparse_mask_workspace_bytes(ho, wo, ctypes.byref(out)), "sparse_mask_workspace_bytes")
    return int(out.value)


def sparse_mask_generate(score: torch.Tensor, ho: int, wo: int, sparsity: float, mask: Optional[torch.Tensor] = None,
                         workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Mask [ho, wo] (uint8, 1 = keep) of one layer from the input-resolution score [in_h, in_w] (float32)."""
    if score.dim() != 2 or score.dtype != torch.float32:
        raise ValueError("score must be a 2-D float32 tensor")
    in_h, in_w = score.shape
    if mask is None:
        mask = torch.empty((ho, wo), dtype=torch.uint8, device=score.device)
    if mask.numel() != ho * wo or mask.dtype != torch.uint8:
        raise ValueError("mask must hold ho*wo bytes")
    if workspace is None:
        workspace = torch.empty(max(sparse_mask_workspace_bytes(ho, wo), 8), dtype=torch.uint8, device=score.device)
    _check(lib().sparse_mask_generate(_dev_ptr(score, "score"), in_h, in_w, ho, wo, float(sparsity),
                                      _dev_ptr(mask, "mask"), _dev_ptr(workspace, "workspace"), workspace.numel(),
                                      _stream_handle(stream)), "sparse_mask_generate")
    return mask


def sc_probe_stream_copy(dst: torch.Tensor, src: torch.Tensor, stream=None):
    """Enqueues the library's plain copy kernel (measurement probe)."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise ValueError("copy probe: sizes differ")
    _check(lib().sc_probe_stream_copy(_dev_ptr(dst, "dst"), _dev_ptr(src, "src"), nbytes, _stream_handle(stream)),
           "sc_probe_stream_copy")


def sc_probe_mfma_bf16(iterations: int, workgroups: int, out: torch.Tensor, stream=None) -> float:
    """Enqueues the register-resident MFMA loop (measurement probe); returns its FLOP count."""
    if out.numel() < workgroups * 256 or out.dtype != torch.float32:
        raise ValueError("mfma probe: out must hold workgroups * 256 floats")
    flops = ctypes.c_double()
    _check(lib().sc_probe_mfma_bf16(iterations, workgroups, _dev_ptr(out, "out"), ctypes.byref(flops),
                                    _stream_handle(stream)), "sc_probe_mfma_bf16")
    return float(flops.value)


SC_STATIC_MASK_PIXELS = 1 << 18


def sparse_mask_generate_static(score: torch.Tensor, ho: int, wo: int, sparsity: float, mask: torch.Tensor,
                                stream=None) -> torch.Tensor:
    """sparse_mask_generate without a workspace: the library's fixed scratch array holds the keys.  The caller
    passes the output tensor; nothing is allocated here or in the library."""
    if score.dim() != 2 or score.dtype != torch.float32:
        raise ValueError("score must be a 2-D float32 tensor")
    in_h, in_w = score.shape
    if mask.numel() != ho * wo or mask.dtype != torch.uint8:
        raise ValueError("mask must hold ho*wo bytes")
    _check(lib().sparse_mask_generate_static(_dev_ptr(score, "score"), in_h, in_w, ho, wo, float(sparsity),
                                             _dev_ptr(mask, "mask"), _stream_handle(stream)),
           "sparse_mask_generate_static")
    return mask


class BackwardPlan:
    """Owner of an sc_bwd_plan handle, its workspace and the forward plan it follows."""

    def __init__(self, handle: int, fwd: Plan, workspace: torch.Tensor):
        self.handle, self.fwd, self.workspace = handle, fwd, workspace

    def close(self):
        if self.handle:
            lib().sparse_conv_backward_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def sparse_conv_backward_workspace_bytes(desc: sc_conv_desc) -> int:
    out = ctypes.c_size_t()
    _check(lib().sparse_conv_backward_workspace_bytes(ctypes.byref(desc), ctypes.byref(out)),
           "sparse_conv_backward_workspace_bytes")
    return int(out.value)


def sparse_conv_backward_plan(fwd: Plan, w: torch.Tensor, workspace: Optional[torch.Tensor] = None, stream=None) -> BackwardPlan:
    d = fwd.desc
    if _CODE_OF_TORCH.get(w.dtype) != d.dtype or w.numel() != d.c_out * d.kh * d.kw * (d.c_in // d.groups):
        raise ValueError("filters do not match the plan")
    nbytes = sparse_conv_backward_workspace_bytes(d)
    if workspace is None:
        workspace = torch.empty(nbytes, dtype=torch.uint8, device=w.device)
    out = ctypes.c_void_p()
    _check(lib().sparse_conv_backward_plan(fwd.handle, ctypes.byref(d), _dev_ptr(w, "w"), _dev_ptr(workspace, "workspace"),
                                           workspace.numel(), _stream_handle(stream), ctypes.byref(out)),
           "sparse_conv_backward_plan")
    return BackwardPlan(out.value, fwd, workspace)


def sparse_conv_backward_set_filters(plan: BackwardPlan, w: torch.Tensor, stream=None):
    d = plan.fwd.desc
    if _CODE_OF_TORCH.get(w.dtype) != d.dtype or w.numel() != d.c_out * d.kh * d.kw * (d.c_in // d.groups):
        raise ValueError("filters do not match the plan")
    _check(lib().sparse_conv_backward_set_filters(plan.handle, _dev_ptr(w, "w"), _stream_handle(stream)),
           "sparse_conv_backward_set_filters")


def sparse_conv_backward_run(plan: BackwardPlan, x: Optional[torch.Tensor], y: Optional[torch.Tensor], dy: torch.Tensor,
                             dx: Optional[torch.Tensor] = None, dw: Optional[torch.Tensor] = None,
                             db: Optional[torch.Tensor] = None, stream=None):
    """Gradients into the tensors given (each optional): dx like x, dw float32 [Cout, kh, kw, Cin], db float32 [Cout]."""
    d = plan.fwd.desc
    info = sparse_conv_plan_info(plan.fwd)
    n_x, n_y = d.n * d.h * d.w * d.c_in, info["m"] * d.c_out
    for t, what, want in ((x, "x", n_x), (dx, "dx", n_x), (y, "y", n_y), (dy, "dy", n_y)):
        if t is not None and (_CODE_OF_TORCH.get(t.dtype) != d.dtype or t.numel() != want):
            raise ValueError(f"{what} does not match the plan")
    if dw is not None and (dw.dtype != torch.float32 or dw.numel() != d.c_out * d.kh * d.kw * d.c_in):
        raise ValueError("dw must be float32 [Cout, kh, kw, Cin]")
    if db is not None and (db.dtype != torch.float32 or db.numel() != d.c_out):
        raise ValueError("db must be float32 [Cout]")
    _check(lib().sparse_conv_backward_run(plan.handle, _dev_ptr(x, "x"), _dev_ptr(y, "y"), _dev_ptr(dy, "dy"),
                                          _dev_ptr(dx, "dx"), _dev_ptr(dw, "dw"), _dev_ptr(db, "db"),
                                          _stream_handle(stream)), "sparse_conv_backward_run")


def prepared_backward_run(plan: BackwardPlan, x, y, dy, dx=None, dw=None, db=None, stream=None):
    """Validate once, run once, and return a zero-argument callable that issues the same backward run again."""
    sparse_conv_backward_run(plan, x, y, dy, dx, dw, db, stream)
    fn, h, st = lib().sparse_conv_backward_run, plan.handle, _stream_handle(stream)
    ptr = lambda t: None if t is None else t.data_ptr()
    args = (ptr(x), ptr(y), ptr(dy), ptr(dx), ptr(dw), ptr(db))
    keep = (plan, x, y, dy, dx, dw, db)

    def call(stream_handle=None):
        rc = fn(h, *args, st if stream_handle is None else stream_handle)
        if rc != SC_OK:
            raise ScError(rc, "sparse_conv_backward_run")
        return keep

    return call
