"""The tiled kernel run as persistent workgroups that share the K steps of all output tiles evenly
(SC_OPT_STREAM_K) against the oracle: tiles finished by one workgroup and tiles completed from partial
sums, every tile shape, ragged tiles, strides, shortcuts, compact operands, repeated launches."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import oracle
from paper_2309_06626_amd import binding as B
from paper_2309_06626_amd import runtime as R
from parity import TOL, assert_close, check_layer, rows_view
from test_gpu_parity import spec_of
from test_gpu_residual import check as check_residual

pytestmark = pytest.mark.gpu

CASES = [
    dict(n=2, cin=128, h=14, w=14, cout=128),                         # 18 K tiles, few output tiles
    dict(n=1, cin=128, h=20, w=17, cout=256, sp=0.3),                 # two channel tiles, ragged row tile
    dict(n=2, cin=256, h=9, w=9, cout=160, sp=0.6),                   # ragged channel tile, 36 K tiles
    dict(n=1, cin=512, h=7, w=7, cout=512, sp=0.5),                   # the deepest ResNet18 shape: 72 K tiles
    dict(n=2, cin=128, h=15, w=15, cout=128, k=3, s=2, p=1, sp=0.4),  # stride 2
    dict(n=4, cin=1024, h=8, w=8, cout=128, k=1, p=0, sp=0.5),        # pointwise with a long K
    dict(n=2, cin=64, h=12, w=12, cout=128, k=5, p=2, d=1, sp=0.5),   # 5x5 window, one K tile per tap
    dict(n=2, cin=128, h=12, w=12, cout=128, k=3, p=2, d=2, sp=0.5),  # dilation 2
]


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("wgs", [8, 24, 64, 512])
@pytest.mark.parametrize("case", range(len(CASES)))
def test_stream_k_kernel(case, wgs, dtype):
    """8 workgroups: each walks several tiles (whole tiles in the middle of its range, a shared tile at either
    end); many workgroups: every tile is completed from several partial sums."""
    spec = spec_of(dtype=dtype, **CASES[case])
    layer = check_layer(W.make_conv_inputs(spec, 1300 + case), tiles=(64, 128), stream_k=wgs)
    assert B.sparse_conv_plan_kernel(layer.plan, 0) == "tile_stream_k"
    tm, tn, got = B.sparse_conv_plan_tiles(layer.plan, 0)
    steps = -(-layer.info["kept"] // 64) * -(-spec.c_out // 128) * (spec.k // 64)
    assert (tm, tn) == (64, 128) and got % 8 == 0 and 8 <= got <= min(wgs, steps // 4)


@pytest.mark.parametrize("tile", [(128, 128), (64, 128), (128, 64), (64, 64)])
@pytest.mark.parametrize("wgs", [16, 40])
def test_stream_k_every_tile_shape(tile, wgs):
    spec = spec_of(2, 256, 12, 12, 160, dtype="bf16", sp=0.4)        # 36 K tiles, ragged rows and channels
    layer = check_layer(W.make_conv_inputs(spec, 1320), tiles=tile, stream_k=wgs)
    assert B.sparse_conv_plan_kernel(layer.plan, 0) == "tile_stream_k"
    steps = -(-layer.info["kept"] // tile[0]) * -(-spec.c_out // tile[1]) * (spec.k // 64)
    assert B.sparse_conv_plan_tiles(layer.plan, 0) == (tile[0], tile[1], min(wgs, steps // 4 // 8 * 8))


def test_stream_k_matches_the_ordinary_launch_where_no_tile_is_shared():
    """Workgroup ranges that end on tile boundaries: no partial sums, the same K order, the same bits."""
    spec = spec_of(2, 128, 16, 16, 128, dtype="bf16", sp=0.5)        # 256 kept rows: 4 tiles of 64 x 128, 18 K tiles
    ci = W.make_conv_inputs(spec, 1321)
    layer = R.ConvLayer(spec, ci.w, ci.bias, ci.mask)
    B.sparse_conv_plan_set_tiles(layer.plan, 0, 64, 128)
    B.sparse_conv_plan_set_tiles(layer.plan, 1, 64, 128)
    x = R.to_device(ci.x, spec.dtype)
    plain_s, plain_d = R.bits_of(layer.sparse(x)).copy(), R.bits_of(layer.dense(x)).copy()
    B.sparse_conv_plan_set_option(layer.plan, B.SC_OPT_STREAM_K, 8)
    assert B.sparse_conv_plan_kernel(layer.plan, 1) == "tile_stream_k"
    assert np.array_equal(R.bits_of(layer.dense(x)), plain_d)        # 8 tiles on 8 workgroups
    B.sparse_conv_plan_set_option(layer.plan, B.SC_OPT_STREAM_K, 1)
    assert B.sparse_conv_plan_kernel(layer.plan, 0) == "tile_lds_direct"
    assert np.array_equal(R.bits_of(layer.sparse(x)), plain_s)


def test_stream_k_repeated_launches_leave_the_counters_clean():
    spec = spec_of(2, 256, 10, 10, 256, dtype="bf16", sp=0.5)
    ci = W.make_conv_inputs(spec, 1322)
    layer = R.ConvLayer(spec, ci.w, ci.bias, ci.mask)
    for which in (0, 1):
        B.sparse_conv_plan_set_tiles(layer.plan, which, 64, 128)
    B.sparse_conv_plan_set_option(layer.plan, B.SC_OPT_STREAM_K, 24)
    assert B.sparse_conv_plan_kernel(layer.plan, 0) == "tile_stream_k" == B.sparse_conv_plan_kernel(layer.plan, 1)
    x = R.to_device(ci.x, spec.dtype)
    first_s = R.bits_of(layer.sparse(x)).copy()
    first_d = R.bits_of(layer.dense(x)).copy()
    for _ in range(20):
        assert np.array_equal(R.bits_of(layer.sparse(x)), first_s)
        assert np.array_equal(R.bits_of(layer.dense(x)), first_d)


def test_stream_k_full_size_deep_layers_sampled_rows():
    """The deepest detector and ResNet18 layers at their full sizes, 512 persistent workgroups."""
    for spec in (spec_of(16, 512, 20, 20, 512, dtype="bf16", sp=0.3, name="y8"),
                 spec_of(64, 256, 14, 14, 256, dtype="bf16", sp=0.5, name="l3"),
                 spec_of(64, 512, 7, 7, 512, dtype="bf16", sp=0.5, name="l4")):
        layer = check_layer(W.make_conv_inputs(spec, 1323), tiles=(64, 128), stream_k=512, sample_rows=256)
        assert B.sparse_conv_plan_kernel(layer.plan, 0) == "tile_stream_k"
        del layer
        torch.cuda.empty_cache()


@pytest.mark.parametrize("post_relu", [False, True])
def test_stream_k_with_a_fused_shortcut(post_relu):
    spec = spec_of(2, 256, 10, 10, 256, dtype="bf16", sp=0.5, relu=False)
    layer = check_residual(spec, 1324, post_relu, want_kernel=("tile_stream_k",), stream_k=24)
    assert B.sparse_conv_plan_tiles(layer.plan, 0) == (64, 128, 24)


def test_stream_k_with_compact_rows():
    spec = spec_of(4, 1024, 8, 8, 128, k=1, p=0, dtype="bf16", sp=0.5)
    ci = W.make_conv_inputs(spec, 1325)
    layer = R.ConvLayer(spec, ci.w, ci.bias, ci.mask)
    B.sparse_conv_plan_set_tiles(layer.plan, 0, 64, 128)
    x = R.to_device(ci.x, "bf16")
    rows = B.plan_row_idx(layer.plan).long()
    xc = x.reshape(spec.m, spec.c_in)[rows].contiguous()
    yc = torch.empty((layer.info["kept"], spec.c_out), dtype=torch.bfloat16, device="cuda:0")
    B.sparse_conv_run_rows(layer.plan, xc, layer.bias, yc, B.SC_ROWS_COMPACT, B.SC_ROWS_COMPACT)
    plain = R.bits_of(yc).copy()
    B.sparse_conv_plan_set_option(layer.plan, B.SC_OPT_STREAM_K, 16)
    yc.fill_(float("nan"))
    B.sparse_conv_run_rows(layer.plan, xc, layer.bias, yc, B.SC_ROWS_COMPACT, B.SC_ROWS_COMPACT)
    torch.cuda.synchronize()
    got = R.to_host_f32(yc)
    ref, absum = oracle.masked_conv2d(spec, ci.x, ci.w, ci.bias, ci.mask, want_absum=True)
    kept = ci.mask == 1
    assert_close(got, rows_view(spec, ref)[kept], rows_view(spec, absum)[kept], TOL["bf16"], "stream-K compact")
    assert plain.shape == R.bits_of(yc).shape
