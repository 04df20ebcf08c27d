"""Compact row formats through the C ABI (sparse_conv_run_rows) against the oracle: the kept rows of a
layer's output as a matrix [kept, Cout], and a pointwise layer reading the kept rows of its input."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import oracle
from paper_2309_06626_amd import binding as B
from paper_2309_06626_amd import runtime as R
from parity import TOL, assert_close, row_mask, rows_view

pytestmark = pytest.mark.gpu

PAD_ROWS = 3   # poisoned rows behind a compact output: nothing may be written past row kept - 1


def layer_spec(name, n, c_in, hw, c_out, k=3, s=1, p=None, dtype="bf16", sparsity=0.5, relu=True, mask_mode="row", w=None):
    p = k // 2 if p is None else p
    return W.ConvSpec(name, n=n, c_in=c_in, h=hw, w=hw if w is None else w, c_out=c_out, kh=k, kw=k, stride_h=s,
                      stride_w=s, pad_h=p, pad_w=p, dtype=dtype, relu=relu, sparsity=sparsity, mask_mode=mask_mode)


def compact_buffer(rows, c, dtype, device="cuda:0"):
    t = torch.empty((rows + PAD_ROWS, c), dtype=B.TORCH_DTYPE[dtype], device=device)
    t.fill_(float("nan"))
    return t


def run_compact_out(layer, x_dev, x_rows=B.SC_ROWS_DENSE):
    spec, kept = layer.spec, layer.info["kept"]
    buf = compact_buffer(kept, spec.c_out, spec.dtype)
    B.sparse_conv_run_rows(layer.plan, x_dev, layer.bias, buf[:kept], x_rows, B.SC_ROWS_COMPACT)
    torch.cuda.synchronize()
    tail = R.to_host_f32(buf[kept:])
    assert np.isnan(tail).all(), "wrote past the last compact row"
    return R.to_host_f32(buf[:kept]), R.bits_of(buf[:kept])


def check_compact_output(spec, seed, tiles=None, gather_pipeline=None, split_k=None, row_panel=None, want_kernel=None):
    ci = W.make_conv_inputs(spec, seed)
    layer = R.ConvLayer(spec, ci.w, ci.bias, ci.mask)
    if tiles is not None:
        B.sparse_conv_plan_set_tiles(layer.plan, 0, *tiles)
    if gather_pipeline is not None:
        B.sparse_conv_plan_set_option(layer.plan, B.SC_OPT_GATHER_PIPELINE, gather_pipeline)
    if split_k is not None:
        B.sparse_conv_plan_set_option(layer.plan, B.SC_OPT_SPLIT_K, split_k)
    if row_panel is not None:
        B.sparse_conv_plan_set_option(layer.plan, B.SC_OPT_ROW_PANEL, row_panel)
    rm = row_mask(spec, ci.mask)
    x = R.to_device(ci.x, spec.dtype)
    got, bits = run_compact_out(layer, x)
    ref, absum = oracle.masked_conv2d(spec, ci.x, ci.w, ci.bias, ci.mask, want_absum=True)
    want = oracle.masked_conv2d_compact(spec, ci.x, ci.w, ci.bias, ci.mask, y_compact=True)
    assert got.shape == want.shape == (int(rm.sum()), spec.c_out)
    assert_close(got, want, oracle.to_compact(absum, rm), TOL[spec.dtype], f"{spec.name} compact out")
    # the dense-layout run of the same plan holds the same numbers at the kept positions, bit for bit
    y = layer.new_output(fill_nan=True)
    layer.sparse(x, y)
    torch.cuda.synchronize()
    kernel = B.sparse_conv_plan_kernel(layer.plan, 0)
    if want_kernel is not None:
        assert want_kernel in kernel
    if "band" not in kernel:          # same kernel, same order of additions
        assert np.array_equal(rows_view(spec, R.bits_of(y))[rm == 1], bits)
    return layer, ci


@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
def test_compact_output_of_a_3x3_layer(dtype):
    # 64 channels at 20x20: the dense-layout run of the 16-bit types takes the band kernel, the compact run a tiled one
    check_compact_output(layer_spec("c3", 3, 64, 20, 64, dtype=dtype, sparsity=0.4), 101,
                         want_kernel=None if dtype == "f32" else "band")


@pytest.mark.parametrize("shape", [
    dict(n=2, c_in=128, hw=14, c_out=256),                       # buffer-load tiled kernel, 32x128 tile
    dict(n=2, c_in=64, hw=28, c_out=128, s=2),                   # strided
    dict(n=1, c_in=24, hw=17, c_out=40),                         # 16-byte gathers through registers, ragged channel tile
    dict(n=2, c_in=5, hw=9, c_out=7),                            # element gather, scalar stores
    dict(n=1, c_in=3, hw=32, c_out=64, k=7, s=2, p=3),           # row-segment gather (stem)
    dict(n=2, c_in=96, hw=12, c_out=64, k=1, p=0),               # pointwise
])
@pytest.mark.parametrize("sparsity", [0.25, 0.7])
def test_compact_output_across_gather_kernels(shape, sparsity):
    check_compact_output(layer_spec("cx", sparsity=sparsity, **shape), 103)


def test_compact_output_with_forced_tiles_pipelines_and_split_k():
    spec = layer_spec("ct", 2, 128, 16, 256, sparsity=0.5)
    for tiles in [(128, 128), (128, 64), (96, 128), (64, 128), (64, 64), (32, 128)]:
        check_compact_output(spec, 107, tiles=tiles)
    check_compact_output(spec, 107, gather_pipeline=1)
    check_compact_output(spec, 107, gather_pipeline=2)
    check_compact_output(spec, 107, tiles=(64, 128), split_k=3)


def test_compact_output_of_the_row_panel_kernel():
    spec = layer_spec("cp", 16, 32, 64, 192, k=1, p=0, sparsity=0.5)      # 32 768 kept rows, one K tile
    layer, _ = check_compact_output(spec, 109, row_panel=2)
    assert B.sparse_conv_plan_kernel(layer.plan, 0) == "tile_row_panel"


def test_spatial_mask_and_degenerate_counts():
    check_compact_output(layer_spec("cs", 3, 64, 10, 64, sparsity=0.5, mask_mode="spatial"), 113)
    for s in (0.0, 0.993):       # every row kept (compact == dense) and a single kept row
        check_compact_output(layer_spec("cd", 1, 16, 12, 32, sparsity=s), 127)
    # no kept row at all: nothing is written, nothing faults
    spec = layer_spec("c0", 1, 16, 8, 16, sparsity=0.5)
    ci = W.make_conv_inputs(spec, 131)
    layer = R.ConvLayer(spec, ci.w, ci.bias, np.zeros_like(ci.mask), check_count=False)
    assert layer.info["kept"] == 0
    buf = compact_buffer(0, spec.c_out, spec.dtype)
    x = R.to_device(ci.x, spec.dtype)
    stream = torch.cuda.current_stream().cuda_stream
    # (an empty tensor has no address: the call goes through the raw entry point with the buffer's own)
    assert B.lib().sparse_conv_run_rows(layer.plan.handle, x.data_ptr(), B.SC_ROWS_DENSE, layer.bias.data_ptr(),
                                        buf.data_ptr(), B.SC_ROWS_COMPACT, stream) == B.SC_OK
    torch.cuda.synchronize()
    assert np.isnan(R.to_host_f32(buf)).all()


@pytest.mark.parametrize("shape,opts", [
    (dict(n=2, c_in=96, hw=12, c_out=64), {}),
    (dict(n=2, c_in=128, hw=14, c_out=256), {}),                          # buffer-load kernel
    (dict(n=2, c_in=128, hw=14, c_out=256), dict(gather_pipeline=1)),     # through registers
    (dict(n=2, c_in=128, hw=14, c_out=256), dict(gather_pipeline=2)),     # global -> LDS
    (dict(n=1, c_in=20, hw=9, c_out=12), {}),                             # element gather
    (dict(n=1, c_in=20, hw=10, c_out=12), {}),                            # element gather, rows of 8-element multiples
    (dict(n=16, c_in=32, hw=64, c_out=192), dict(row_panel=2)),           # row panel
    (dict(n=2, c_in=64, hw=10, c_out=32, dtype="f32"), {}),
    (dict(n=2, c_in=64, hw=10, c_out=32, dtype="f16"), {}),
])
def test_pointwise_layer_reads_compact_input(shape, opts):
    spec = layer_spec("px", k=1, p=0, sparsity=0.45, **shape)
    ci = W.make_conv_inputs(spec, 137)
    layer = R.ConvLayer(spec, ci.w, ci.bias, ci.mask)
    for name, opt in (("gather_pipeline", B.SC_OPT_GATHER_PIPELINE), ("row_panel", B.SC_OPT_ROW_PANEL)):
        if name in opts:
            B.sparse_conv_plan_set_option(layer.plan, opt, opts[name])
    rm = row_mask(spec, ci.mask)
    xc_host = oracle.to_compact(ci.x, rm)                        # the producer's compact rows
    xc = R.to_device(xc_host, spec.dtype)
    ref_dense, absum = oracle.masked_conv2d(spec, oracle.from_compact(xc_host, rm, spec.x_shape()), ci.w, ci.bias,
                                            ci.mask, want_absum=True)
    tol = TOL[spec.dtype]
    # compact in, dense out: kept rows placed, dropped rows zero
    y = layer.new_output(fill_nan=True)
    B.sparse_conv_run_rows(layer.plan, xc, layer.bias, y, B.SC_ROWS_COMPACT, B.SC_ROWS_DENSE)
    torch.cuda.synchronize()
    g, bits = rows_view(spec, R.to_host_f32(y)), rows_view(spec, R.bits_of(y))
    assert (bits[rm == 0] == 0).all()
    want = oracle.masked_conv2d_compact(spec, xc_host, ci.w, ci.bias, ci.mask, x_compact=True)
    assert_close(g[rm == 1], rows_view(spec, want)[rm == 1], rows_view(spec, absum)[rm == 1], tol, "compact in, dense out")
    # compact in, compact out: a plain GEMM over the kept rows
    got, cbits = run_compact_out(layer, xc, B.SC_ROWS_COMPACT)
    want_c = oracle.masked_conv2d_compact(spec, xc_host, ci.w, ci.bias, ci.mask, x_compact=True, y_compact=True)
    assert_close(got, want_c, oracle.to_compact(absum, rm), tol, "compact in, compact out")
    assert np.array_equal(cbits, bits[rm == 1])
    # and the ordinary run on the expanded input gives the same bits
    y2 = layer.new_output(fill_nan=True)
    layer.sparse(R.to_device(oracle.from_compact(xc_host, rm, spec.x_shape()), spec.dtype), y2)
    torch.cuda.synchronize()
    assert np.array_equal(R.bits_of(y2), R.bits_of(y))


def test_chain_of_layers_that_share_a_mask_stays_compact():
    """3x3 (dense in, compact out) -> 1x1 (compact, compact) -> 1x1 (compact in, dense out): one 2-D mask
    for the whole resolution, as the propagated masks of Sec. 3.1 give; the result equals the chain
    in which every layer writes its dense map."""
    n, hw, dtype = 4, 28, "bf16"
    specs = [layer_spec("a", n, 64, hw, 128, k=3, mask_mode="spatial", dtype=dtype),
             layer_spec("b", n, 128, hw, 256, k=1, p=0, mask_mode="spatial", dtype=dtype),
             layer_spec("c", n, 256, hw, 64, k=1, p=0, mask_mode="spatial", dtype=dtype)]
    mask = W.gen_mask(hw * hw, W.n_keep(0.5, hw * hw), 211)
    cis = [W.make_conv_inputs(s.with_(layer_index=i), 223) for i, s in enumerate(specs)]
    layers = [R.ConvLayer(s, ci.w, ci.bias, mask) for s, ci in zip(specs, cis)]
    x_host = cis[0].x
    # oracle: the dense chain, every output rounded to the storage type
    t = x_host
    for s, ci in zip(specs, cis):
        t = oracle.round_storage(oracle.masked_conv2d(s, t, ci.w, ci.bias, mask), dtype)
    ref = t
    kept = layers[0].info["kept"]
    a = torch.empty((kept, 128), dtype=B.TORCH_DTYPE[dtype], device="cuda:0").fill_(float("nan"))
    b = torch.empty((kept, 256), dtype=B.TORCH_DTYPE[dtype], device="cuda:0").fill_(float("nan"))
    y = layers[2].new_output(fill_nan=True)
    B.sparse_conv_run_rows(layers[0].plan, R.to_device(x_host, dtype), layers[0].bias, a, B.SC_ROWS_DENSE, B.SC_ROWS_COMPACT)
    B.sparse_conv_run_rows(layers[1].plan, a, layers[1].bias, b, B.SC_ROWS_COMPACT, B.SC_ROWS_COMPACT)
    B.sparse_conv_run_rows(layers[2].plan, b, layers[2].bias, y, B.SC_ROWS_COMPACT, B.SC_ROWS_DENSE)
    torch.cuda.synchronize()
    g = R.to_host_f32(y)
    rm = np.tile(mask, n)
    assert (rows_view(specs[2], R.bits_of(y))[rm == 0] == 0).all()
    nr = np.linalg.norm(ref.astype(np.float64))
    assert np.linalg.norm(g.astype(np.float64) - ref) / nr <= TOL[dtype]
    assert np.abs(g - ref).max() <= TOL[dtype] * np.abs(ref).max()
    # the all-dense-layout chain on the GPU agrees with the compact chain bit for bit
    t = R.to_device(x_host, dtype)
    for layer in layers:
        t = layer.sparse(t)
    torch.cuda.synchronize()
    assert np.array_equal(R.bits_of(t), R.bits_of(y))


def test_compact_formats_that_make_no_sense_are_refused():
    spec = layer_spec("e", 1, 16, 8, 16)
    ci = W.make_conv_inputs(spec, 307)
    layer = R.ConvLayer(spec, ci.w, ci.bias, ci.mask)
    kept = layer.info["kept"]
    x = R.to_device(ci.x, spec.dtype)
    xc = torch.zeros((kept, 16), dtype=torch.bfloat16, device="cuda:0")
    y = layer.new_output()
    L = B.lib()
    args = (layer.plan.handle, xc.data_ptr(), B.SC_ROWS_COMPACT, layer.bias.data_ptr(), y.data_ptr(), B.SC_ROWS_DENSE, None)
    assert L.sparse_conv_run_rows(*args) == B.SC_ERR_UNSUPPORTED            # a 3x3 window reads dropped neighbours
    assert L.sparse_conv_run_rows(layer.plan.handle, x.data_ptr(), 2, layer.bias.data_ptr(), y.data_ptr(), 0, None) == B.SC_ERR_UNSUPPORTED
    assert L.sparse_conv_run_rows(layer.plan.handle, x.data_ptr(), 0, layer.bias.data_ptr(), y.data_ptr(), -1, None) == B.SC_ERR_UNSUPPORTED
    assert L.sparse_conv_run_rows(None, x.data_ptr(), 0, None, y.data_ptr(), 0, None) == B.SC_ERR_NULL
    spec_n = layer_spec("en", 1, 16, 8, 16).with_(layout="nchw")
    cin = W.make_conv_inputs(spec_n, 311)
    layer_n = R.ConvLayer(spec_n, cin.w, cin.bias, cin.mask)
    yn = layer_n.new_output()
    xn = R.to_device(cin.x, spec_n.dtype)
    assert L.sparse_conv_run_rows(layer_n.plan.handle, xn.data_ptr(), 0, layer_n.bias.data_ptr(), yn.data_ptr(), 1, None) == B.SC_ERR_UNSUPPORTED
    # the binding refuses operands of the wrong size before the library sees them
    with pytest.raises(ValueError):
        B.sparse_conv_run_rows(layer.plan, x, layer.bias, y[:, :3], B.SC_ROWS_DENSE, B.SC_ROWS_COMPACT)
    # dense formats on both sides are the ordinary run
    y1, y2 = layer.new_output(fill_nan=True), layer.new_output(fill_nan=True)
    B.sparse_conv_run_rows(layer.plan, x, layer.bias, y1)
    layer.sparse(x, y2)
    torch.cuda.synchronize()
    assert np.array_equal(R.bits_of(y1), R.bits_of(y2))
