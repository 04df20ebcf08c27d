"""Masked depthwise layers (groups == Cin == Cout) through the C ABI against the oracle."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import oracle
from paper_2309_06626_amd import binding as B
from paper_2309_06626_amd import runtime as R
from parity import TOL, assert_close, row_mask, rows_view

pytestmark = pytest.mark.gpu


def dw_spec(n, c, h, w, k=3, s=1, p=None, d=1, dtype="bf16", sparsity=0.5, relu=True, bias=True, mask_mode="row"):
    p = (d * (k - 1)) // 2 if p is None else p
    return W.ConvSpec("dw", n=n, c_in=c, h=h, w=w, c_out=c, kh=k, kw=k, stride_h=s, stride_w=s, pad_h=p, pad_w=p,
                      dil_h=d, dil_w=d, dtype=dtype, has_bias=bias, relu=relu, sparsity=sparsity, mask_mode=mask_mode,
                      groups=c)


def check_depthwise(spec, seed, out_mode=B.SC_OUT_ZERO_FILL):
    ci = W.make_conv_inputs(spec, seed)
    assert ci.w.shape == (spec.c_out, spec.kh, spec.kw, 1)
    layer = R.ConvLayer(spec, ci.w, ci.bias, ci.mask, out_mode=out_mode)
    assert B.sparse_conv_plan_kernel(layer.plan, 0) == "depthwise"
    rm = row_mask(spec, ci.mask)
    assert np.array_equal(B.plan_row_idx(layer.plan).cpu().numpy(), oracle.compact_rows(rm))
    tol = TOL[spec.dtype]
    x = R.to_device(ci.x, spec.dtype)
    ref, absum = oracle.masked_depthwise_conv2d(spec, ci.x, ci.w, ci.bias, ci.mask, want_absum=True)
    ref, absum = rows_view(spec, ref), rows_view(spec, absum)
    kept = rm == 1
    # dense layout
    sentinel = float("nan") if out_mode == B.SC_OUT_ZERO_FILL else 7.0
    y = layer.new_output()
    y.fill_(sentinel)
    layer.sparse(x, y)
    torch.cuda.synchronize()
    g, bits = rows_view(spec, R.to_host_f32(y)), rows_view(spec, R.bits_of(y))
    if out_mode == B.SC_OUT_ZERO_FILL:
        assert (bits[~kept] == 0).all(), "dropped pixels must be +0.0 in every channel"
    else:
        assert (g[~kept] == 7.0).all(), "scatter-only mode must not touch dropped pixels"
    assert_close(g[kept], ref[kept], absum[kept], tol, "depthwise sparse")
    # compact output: the same bits, nothing written behind the last kept row
    n_kept = int(kept.sum())
    buf = torch.empty((n_kept + 2, spec.c_out), dtype=B.TORCH_DTYPE[spec.dtype], device="cuda:0").fill_(float("nan"))
    if n_kept:
        B.sparse_conv_run_rows(layer.plan, x, layer.bias, buf[:n_kept], B.SC_ROWS_DENSE, B.SC_ROWS_COMPACT)
        torch.cuda.synchronize()
        assert np.array_equal(R.bits_of(buf[:n_kept]), bits[kept])
    assert np.isnan(R.to_host_f32(buf[n_kept:])).all()
    # dense run: the mask is ignored
    yd = layer.new_output(fill_nan=True)
    layer.dense(x, yd)
    torch.cuda.synchronize()
    refd, absd = oracle.masked_depthwise_conv2d(spec, ci.x, ci.w, ci.bias, np.ones_like(ci.mask), want_absum=True)
    assert_close(rows_view(spec, R.to_host_f32(yd)), rows_view(spec, refd), rows_view(spec, absd), tol, "depthwise dense")
    assert np.array_equal(rows_view(spec, R.bits_of(yd))[kept], bits[kept])
    return layer


@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
@pytest.mark.parametrize("shape", [
    dict(n=2, c=32, h=14, w=14),                       # 16-byte channel groups
    dict(n=1, c=96, h=17, w=11, s=2),                  # stride 2, ragged map
    dict(n=2, c=20, h=9, w=9),                         # 16-byte groups for float only
    dict(n=1, c=7, h=8, w=10),                         # one channel per lane
    dict(n=1, c=16, h=12, w=12, k=5),                  # 5x5 window
    dict(n=1, c=8, h=13, w=13, d=2),                   # dilation 2
    dict(n=2, c=24, h=6, w=6, k=1),                    # 1x1: a per-channel scale
])
def test_depthwise_layers(dtype, shape):
    check_depthwise(dw_spec(dtype=dtype, sparsity=0.4, **shape), 401)


@pytest.mark.parametrize("sparsity", [0.0, 0.25, 0.7])
def test_depthwise_sparsities_and_modes(sparsity):
    spec = dw_spec(2, 64, 20, 20, sparsity=sparsity)
    check_depthwise(spec, 409)
    check_depthwise(spec, 409, out_mode=B.SC_OUT_SCATTER_ONLY)
    check_depthwise(dw_spec(3, 32, 10, 10, sparsity=sparsity if sparsity else 0.5, mask_mode="spatial"), 419)
    check_depthwise(dw_spec(1, 16, 9, 9, sparsity=0.3, relu=False, bias=False), 421)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("mask_mode", ["row", "spatial"])
@pytest.mark.parametrize("out_mode", [B.SC_OUT_ZERO_FILL, B.SC_OUT_SCATTER_ONLY])
def test_pointwise_depthwise_layer_with_compact_operands(dtype, mask_mode, out_mode):
    """1x1 window, stride 1, no padding: the window is the pixel itself, so the layer takes the kept rows of its
    input as they are.  Every combination of row formats; the compact buffers hold exactly the kept rows plus guard
    rows of NaN that no launch may read from or write to."""
    spec = dw_spec(3, 24, 9, 7, k=1, dtype=dtype, sparsity=0.6, mask_mode=mask_mode)
    ci = W.make_conv_inputs(spec, 461)
    layer = R.ConvLayer(spec, ci.w, ci.bias, ci.mask, out_mode=out_mode)
    rm = row_mask(spec, ci.mask)
    kept = rm == 1
    n_kept = int(kept.sum())
    assert 0 < n_kept < spec.m
    ref, absum = oracle.masked_depthwise_conv2d(spec, ci.x, ci.w, ci.bias, ci.mask, want_absum=True)
    ref, absum = rows_view(spec, ref), rows_view(spec, absum)
    via_compact = oracle.masked_depthwise_conv2d_compact(spec, oracle.to_compact(ci.x, rm), ci.w, ci.bias, ci.mask,
                                                         x_mask=ci.mask, y_compact=True)
    assert np.array_equal(via_compact, ref[kept])
    td = B.TORCH_DTYPE[dtype]
    D, C = B.SC_ROWS_DENSE, B.SC_ROWS_COMPACT
    # the compact input: kept rows, then guard rows whose NaN would show in any result that read them
    xc = torch.empty((n_kept + 3, spec.c_in), dtype=td, device="cuda:0").fill_(float("nan"))
    xc[:n_kept] = R.to_device(np.ascontiguousarray(ci.x.reshape(-1, spec.c_in)[kept]), dtype)
    x = R.to_device(ci.x, dtype)
    tol = TOL[dtype]
    # reference bits: the dense-format run
    sentinel = float("nan") if out_mode == B.SC_OUT_ZERO_FILL else 7.0
    y = layer.new_output()
    y.fill_(sentinel)
    layer.sparse(x, y)
    torch.cuda.synchronize()
    bits = rows_view(spec, R.bits_of(y))
    assert_close(rows_view(spec, R.to_host_f32(y))[kept], ref[kept], absum[kept], tol, "1x1 depthwise")
    # compact in, dense out
    y2 = layer.new_output()
    y2.fill_(sentinel)
    B.sparse_conv_run_rows(layer.plan, xc[:n_kept], layer.bias, y2, C, D)
    torch.cuda.synchronize()
    assert np.array_equal(rows_view(spec, R.bits_of(y2)), bits)
    # dense in, compact out and compact in, compact out: the kept rows and nothing behind them
    for x_in, fmt in ((x, D), (xc[:n_kept], C)):
        buf = torch.empty((n_kept + 3, spec.c_out), dtype=td, device="cuda:0").fill_(float("nan"))
        B.sparse_conv_run_rows(layer.plan, x_in, layer.bias, buf[:n_kept], fmt, C)
        torch.cuda.synchronize()
        assert np.array_equal(R.bits_of(buf[:n_kept]), bits[kept])
        assert np.isnan(R.to_host_f32(buf[n_kept:])).all(), "nothing may be written behind the last kept row"


def test_depthwise_all_rows_dropped():
    spec = dw_spec(1, 16, 8, 8)
    ci = W.make_conv_inputs(spec, 431)
    layer = R.ConvLayer(spec, ci.w, ci.bias, np.zeros_like(ci.mask), check_count=False)
    y = layer.new_output(fill_nan=True)
    layer.sparse(R.to_device(ci.x, spec.dtype), y)
    torch.cuda.synchronize()
    assert (R.bits_of(y) == 0).all()


def test_mobilenet_style_block_with_one_mask_stays_compact_between_pointwise_layers():
    """expand 1x1 -> depthwise 3x3 -> project 1x1 -> next expand 1x1, all at one resolution with one 2-D mask:
    the depthwise layer needs its neighbours, so its input is a dense map; project and the next expand hand
    each other the kept rows only."""
    n, hw, dtype = 2, 28, "bf16"
    mk = dict(dtype=dtype, mask_mode="spatial", sparsity=0.5)
    expand = W.ConvSpec("expand", n=n, c_in=24, h=hw, w=hw, c_out=144, kh=1, kw=1, pad_h=0, pad_w=0, layer_index=0, **mk)
    dw = dw_spec(n, 144, hw, hw, **mk).with_(name="dw", layer_index=1)
    project = W.ConvSpec("project", n=n, c_in=144, h=hw, w=hw, c_out=32, kh=1, kw=1, pad_h=0, pad_w=0, relu=False,
                         layer_index=2, **mk)
    expand2 = W.ConvSpec("expand2", n=n, c_in=32, h=hw, w=hw, c_out=192, kh=1, kw=1, pad_h=0, pad_w=0, layer_index=3, **mk)
    specs = [expand, dw, project, expand2]
    mask = W.gen_mask(hw * hw, W.n_keep(0.5, hw * hw), 443)
    cis = [W.make_conv_inputs(s, 449) for s in specs]
    layers = [R.ConvLayer(s, ci.w, ci.bias, mask) for s, ci in zip(specs, cis)]
    x_host = cis[0].x
    # oracle: every layer in dense layout, outputs rounded to the storage type
    t = x_host
    for s, ci in zip(specs, cis):
        conv = oracle.masked_depthwise_conv2d if s.groups > 1 else oracle.masked_conv2d
        t = oracle.round_storage(conv(s, t, ci.w, ci.bias, mask), dtype)
    ref = t
    kept = layers[0].info["kept"]
    td = B.TORCH_DTYPE[dtype]
    a = layers[0].new_output(fill_nan=True)
    b = layers[1].new_output(fill_nan=True)
    c = torch.empty((kept, 32), dtype=td, device="cuda:0").fill_(float("nan"))
    y = layers[3].new_output(fill_nan=True)
    D, C = B.SC_ROWS_DENSE, B.SC_ROWS_COMPACT
    B.sparse_conv_run_rows(layers[0].plan, R.to_device(x_host, dtype), layers[0].bias, a, D, D)
    B.sparse_conv_run_rows(layers[1].plan, a, layers[1].bias, b, D, D)
    B.sparse_conv_run_rows(layers[2].plan, b, layers[2].bias, c, D, C)
    B.sparse_conv_run_rows(layers[3].plan, c, layers[3].bias, y, C, D)
    torch.cuda.synchronize()
    g = R.to_host_f32(y)
    rm = np.tile(mask, n)
    assert (rows_view(specs[3], R.bits_of(y))[rm == 0] == 0).all()
    nr = np.linalg.norm(ref.astype(np.float64))
    assert np.linalg.norm(g.astype(np.float64) - ref) / nr <= TOL[dtype]
    assert np.abs(g - ref).max() <= TOL[dtype] * np.abs(ref).max()


@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
@pytest.mark.parametrize("stride", [1, 2])
def test_a_non_finite_input_value_reaches_only_the_windows_that_contain_it(dtype, stride):
    """The 16-bit kernels pair window rows with rows outside the window (times a zero filter entry): an
    infinity there must not leak into the result as 0 * inf."""
    spec = dw_spec(1, 16, 12, 12, s=stride, dtype=dtype, sparsity=0.0, relu=False)
    ci = W.make_conv_inputs(spec, 457)
    x = ci.x.copy()
    x[0, 5, 6, :] = np.inf
    x[0, 8, 2, 3] = -np.inf
    layer = R.ConvLayer(spec, ci.w, ci.bias, ci.mask)
    y = layer.new_output(fill_nan=True)
    layer.sparse(R.to_device(x, dtype), y)
    torch.cuda.synchronize()
    got = R.to_host_f32(y)
    with np.errstate(invalid="ignore", over="ignore"):
        ref = oracle.masked_depthwise_conv2d(spec, x, ci.w, ci.bias, ci.mask)
    finite = np.isfinite(ref)
    assert np.array_equal(np.isfinite(got), finite)
    assert finite.sum() < ref.size and not finite.all()
    clean = oracle.masked_depthwise_conv2d(spec, ci.x, ci.w, ci.bias, ci.mask)
    assert np.abs(got[finite] - clean[finite]).max() <= TOL[dtype] * np.abs(clean).max()


# ---------------------------------------------------------------------------------------------------------
# compact input under the producer's mask (sparse_conv_plan_set_input_mask)
# ---------------------------------------------------------------------------------------------------------
def check_compact_input(spec, seed, in_sparsity=0.5):
    ci = W.make_conv_inputs(spec, seed)
    layer = R.ConvLayer(spec, ci.w, ci.bias, ci.mask)
    pixels = spec.h * spec.w
    length = spec.n * pixels if spec.mask_mode == "row" else pixels
    x_mask = W.gen_mask(length, W.n_keep(in_sparsity, length), seed + 2)
    in_rows = x_mask if spec.mask_mode == "row" else np.tile(x_mask, spec.n)
    # a value the window must not see sits at every dropped pixel of the dense map the oracle expands to zeros
    xc_host = np.ascontiguousarray(ci.x.reshape(-1, spec.c_in)[in_rows == 1])
    n_in = xc_host.shape[0]
    assert B.sparse_conv_plan_set_input_mask(layer.plan, torch.from_numpy(x_mask).to("cuda:0")) == n_in
    tol = TOL[spec.dtype]
    xz = ci.x * in_rows.reshape(spec.n, spec.h, spec.w, 1)
    ref, absum = oracle.masked_depthwise_conv2d(spec, xz, ci.w, ci.bias, ci.mask, want_absum=True)
    via_compact = oracle.masked_depthwise_conv2d_compact(spec, xc_host, ci.w, ci.bias, ci.mask, x_mask=x_mask)
    assert np.array_equal(via_compact, ref)
    ref, absum = rows_view(spec, ref), rows_view(spec, absum)
    rm = row_mask(spec, ci.mask)
    kept = rm == 1
    dt = B.TORCH_DTYPE[spec.dtype]
    xc = R.to_device(xc_host, spec.dtype) if n_in else torch.empty((0, spec.c_in), dtype=dt, device="cuda:0")
    y = layer.new_output(fill_nan=True)
    if n_in:
        B.sparse_conv_run_rows(layer.plan, xc, layer.bias, y, B.SC_ROWS_COMPACT, B.SC_ROWS_DENSE)
    else:   # (an empty tensor has no address: the library is called with a placeholder it never reads)
        pad = torch.zeros((1, spec.c_in), dtype=dt, device="cuda:0")
        B._check(B.lib().sparse_conv_run_rows(layer.plan.handle, pad.data_ptr(), B.SC_ROWS_COMPACT,
                                              layer.bias.data_ptr() if layer.bias is not None else None, y.data_ptr(),
                                              B.SC_ROWS_DENSE, None), "sparse_conv_run_rows")
    torch.cuda.synchronize()
    g, bits = rows_view(spec, R.to_host_f32(y)), rows_view(spec, R.bits_of(y))
    assert (bits[~kept] == 0).all()
    assert_close(g[kept], ref[kept], absum[kept], tol, "depthwise, compact input")
    # the dense-layout run on the zero-filled map computes the same numbers
    yz = layer.new_output(fill_nan=True)
    layer.sparse(R.to_device(xz, spec.dtype), yz)
    torch.cuda.synchronize()
    if spec.dtype == "f32":     # (another kernel, another order of the nine products)
        assert_close(rows_view(spec, R.to_host_f32(yz))[kept], g[kept], absum[kept], 2 * tol, "zero-filled map")
    else:
        assert np.array_equal(R.bits_of(yz), R.bits_of(y))
    # compact in, compact out
    n_kept = int(kept.sum())
    if n_kept and n_in:
        buf = torch.empty((n_kept + 1, spec.c_out), dtype=xc.dtype, device="cuda:0").fill_(float("nan"))
        B.sparse_conv_run_rows(layer.plan, xc, layer.bias, buf[:n_kept], B.SC_ROWS_COMPACT, B.SC_ROWS_COMPACT)
        torch.cuda.synchronize()
        assert np.array_equal(R.bits_of(buf[:n_kept]), bits[kept])
        assert np.isnan(R.to_host_f32(buf[n_kept:])).all()
    return layer


@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
@pytest.mark.parametrize("shape", [
    dict(n=2, c=32, h=14, w=14),                       # one tile per image
    dict(n=1, c=96, h=37, w=29, s=2),                  # stride 2: the input mask has another resolution; ragged tiles
    dict(n=3, c=144, h=40, w=40),                      # several tiles per workgroup: ranks are fetched a tile ahead
    dict(n=1, c=576, h=14, w=14),                      # several channel chunks
    dict(n=1, c=7, h=8, w=10),                         # one channel per lane
    dict(n=1, c=16, h=12, w=12, k=5),                  # 5x5 window: the general kernel
    dict(n=1, c=8, h=13, w=13, d=2),                   # dilation 2
])
@pytest.mark.parametrize("mask_mode", ["row", "spatial"])
def test_depthwise_reads_a_compact_input_through_its_producers_mask(dtype, shape, mask_mode):
    check_compact_input(dw_spec(dtype=dtype, sparsity=0.4, mask_mode=mask_mode, **shape), 431)


@pytest.mark.parametrize("in_sparsity", [0.0, 0.9, 1.0])
def test_compact_input_extremes(in_sparsity):
    check_compact_input(dw_spec(2, 64, 18, 18, sparsity=0.5, mask_mode="spatial"), 433, in_sparsity=in_sparsity)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_compact_input_with_a_layer_mask_that_keeps_every_pixel(dtype):
    check_compact_input(dw_spec(2, 24, 15, 15, s=2, sparsity=0.0, dtype=dtype, mask_mode="spatial"), 434)


def test_many_tiles_per_workgroup_with_a_compact_input():
    """A map large enough that every persistent workgroup walks several tiles."""
    check_compact_input(dw_spec(8, 32, 112, 112, sparsity=0.5, mask_mode="spatial"), 435)
    check_compact_input(dw_spec(8, 96, 112, 112, s=2, sparsity=0.5, mask_mode="spatial"), 436)


def test_compact_input_needs_the_input_mask_first_and_only_depthwise_window_layers_take_one():
    spec = dw_spec(1, 16, 10, 10)
    ci = W.make_conv_inputs(spec, 437)
    layer = R.ConvLayer(spec, ci.w, ci.bias, ci.mask)
    x = R.to_device(ci.x, spec.dtype)
    y = layer.new_output()
    rc = B.lib().sparse_conv_run_rows(layer.plan.handle, x.data_ptr(), B.SC_ROWS_COMPACT, layer.bias.data_ptr(),
                                      y.data_ptr(), B.SC_ROWS_DENSE, None)
    assert rc == B.SC_ERR_UNSUPPORTED
    with pytest.raises(ValueError):
        B.sparse_conv_run_rows(layer.plan, x, layer.bias, y, B.SC_ROWS_COMPACT, B.SC_ROWS_DENSE)
    # an ordinary 3x3 layer has no such map
    spec2 = W.ConvSpec("c", n=1, c_in=16, h=10, w=10, c_out=16, dtype="bf16", sparsity=0.5)
    ci2 = W.make_conv_inputs(spec2, 438)
    layer2 = R.ConvLayer(spec2, ci2.w, ci2.bias, ci2.mask)
    m = torch.ones(100, dtype=torch.uint8, device="cuda:0")
    assert B.lib().sparse_conv_plan_set_input_mask(layer2.plan.handle, m.data_ptr(), None, None) == B.SC_ERR_UNSUPPORTED
    assert B.lib().sparse_conv_plan_set_input_mask(layer.plan.handle, None, None, None) == B.SC_ERR_NULL
