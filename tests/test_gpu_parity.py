"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle."""
import ctypes

import numpy as np
import pytest
import torch

import workloads as W
from oracle import oracle
from paper_2309_06626_amd import binding as B
from paper_2309_06626_amd import runtime as R
from parity import TOL, assert_close, check_layer, compare_network, rows_view

pytestmark = pytest.mark.gpu

ALL_TILES = [(256, 128), (128, 256), (128, 128), (256, 64), (128, 64), (96, 128), (64, 128), (64, 64), (128, 32), (32, 128)]


def spec_of(n, cin, h, w, cout, k=3, s=1, p=1, d=1, dtype="bf16", layout="nhwc", bias=True, relu=True, sp=0.5,
            mask_mode="row", kw=None, sw=None, pw=None, dw=None, name="t"):
    return W.ConvSpec(name, n=n, c_in=cin, h=h, w=w, c_out=cout, kh=k, kw=k if kw is None else kw, stride_h=s,
                      stride_w=s if sw is None else sw, pad_h=p, pad_w=p if pw is None else pw, dil_h=d,
                      dil_w=d if dw is None else dw, dtype=dtype, layout=layout, has_bias=bias, relu=relu,
                      sparsity=sp, mask_mode=mask_mode)


def test_config1_fp32():
    ci = W.make_conv_inputs(W.config1(), W.base_seed(1))
    assert ci.keep == 128
    check_layer(ci)


SMALL = [
    # several tiles and a ragged tail in M; channel counts off the vector widths; every conv knob
    dict(n=3, cin=16, h=19, w=19, cout=32),
    dict(n=2, cin=24, h=17, w=23, cout=48, sp=0.3),
    dict(n=2, cin=5, h=14, w=11, cout=7, sp=0.4),                      # element gather, ragged channels
    dict(n=1, cin=3, h=37, w=41, cout=64, k=7, s=2, p=3, sp=0.5),      # stem-like
    dict(n=2, cin=32, h=15, w=15, cout=40, k=1, p=0, sp=0.5),          # pointwise
    dict(n=2, cin=16, h=20, w=13, cout=16, k=3, s=2, p=1, sp=0.25),
    dict(n=1, cin=8, h=21, w=18, cout=24, k=3, s=1, p=2, d=2, sp=0.6),
    dict(n=2, cin=8, h=16, w=12, cout=16, k=3, kw=2, s=2, sw=1, p=0, pw=1, d=1, dw=1, sp=0.5),
    dict(n=4, cin=64, h=9, w=9, cout=160, k=1, p=0, s=2, sp=0.5),      # strided pointwise (downsample)
    dict(n=1, cin=16, h=6, w=6, cout=16, sp=0.9),                      # very few rows
]


@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
@pytest.mark.parametrize("layout", ["nhwc", "nchw"])
@pytest.mark.parametrize("case", range(len(SMALL)))
def test_small_layers(case, layout, dtype):
    spec = spec_of(dtype=dtype, layout=layout, **SMALL[case])
    check_layer(W.make_conv_inputs(spec, 500 + case))


@pytest.mark.parametrize("bias,relu", [(False, False), (True, False), (False, True)])
def test_bias_relu_switches(bias, relu):
    spec = spec_of(2, 16, 12, 12, 32, dtype="bf16", bias=bias, relu=relu, sp=0.5)
    check_layer(W.make_conv_inputs(spec, 77))


@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
@pytest.mark.parametrize("tile", ALL_TILES)
def test_every_tile_shape(tile, dtype):
    # kept = 1444 rows: several tiles of every height plus a ragged last tile; Cout = 160 leaves a
    # ragged channel tile for the 64- and 128-wide shapes
    spec = spec_of(8, 32, 19, 19, 160, dtype=dtype, sp=0.5)
    layer = check_layer(W.make_conv_inputs(spec, 31), tiles=tile)
    assert B.sparse_conv_plan_tiles(layer.plan, 0)[:2] == tile


def test_tile_choice_follows_the_reduced_row_count():
    spec = spec_of(16, 72, 28, 28, 128, sp=0.0)    # 72 channels: only the tiled gather kernel applies
    wide = R.ConvLayer(spec, *_wbm(spec, 5))
    spec9 = spec.with_(sparsity=0.9)
    narrow = R.ConvLayer(spec9, *_wbm(spec9, 5))
    tm0, tn0, wg0 = B.sparse_conv_plan_tiles(wide.plan, 0)
    tm1, tn1, wg1 = B.sparse_conv_plan_tiles(narrow.plan, 0)
    assert tm1 * tn1 <= tm0 * tn0
    assert B.sparse_conv_plan_tiles(narrow.plan, 1)[:2] == (tm0, tn0)   # its dense run keeps the wide tile
    with pytest.raises(B.ScError):
        B.sparse_conv_plan_set_tiles(wide.plan, 0, 48, 48)


def test_deep_layer_choice_fills_the_compute_units_in_one_round():
    """The deepest detector layer at s = 0.3: 4 480 kept rows would make 280 tiles of 64 x 128 on 256 compute units (two
    on some, one on the rest).  The priced choice stays within one round of workgroups, and matches the oracle."""
    spec = spec_of(16, 512, 20, 20, 512, dtype="bf16", sp=0.3)
    layer = check_layer(W.make_conv_inputs(spec, 975), sample_rows=256)
    tm, tn, wgs = B.sparse_conv_plan_tiles(layer.plan, 0)
    assert wgs <= 256 and tm * tn >= 96 * 128
    assert B.sparse_conv_plan_kernel(layer.plan, 0) in ("tile_lds_direct", "tile_split_k")


def test_masked_store_variant_matches_the_row_list_variant():
    """A sparse run that contracts every row and applies the mask at the store (small layers): same kernels, same K
    order, so the kept rows carry the bits of the row-list run, and the dropped rows are zeros or untouched."""
    cases = [dict(n=4, cin=192, h=14, w=14, cout=32, k=1, p=0),            # buffer-load form
             dict(n=2, cin=32, h=9, w=11, cout=192, k=1, p=0, sp=0.3),     # direct-to-LDS form, one K tile
             dict(n=1, cin=24, h=13, w=13, cout=40, sp=0.6),                # register-staged form, 16-byte groups only
             dict(n=2, cin=128, h=10, w=10, cout=128, sp=0.5, mask_mode="spatial"),
             dict(n=1, cin=5, h=9, w=8, cout=7, sp=0.5)]                    # element gather and element stores
    for i, case in enumerate(cases):
        for dtype in ("bf16", "f32"):
            for out_mode in (B.SC_OUT_ZERO_FILL, B.SC_OUT_SCATTER_ONLY):
                spec = spec_of(dtype=dtype, **case)
                ci = W.make_conv_inputs(spec, 1100 + i)
                layer = R.ConvLayer(spec, ci.w, ci.bias, ci.mask, out_mode=out_mode)
                B.sparse_conv_plan_set_tiles(layer.plan, 0, 64, 64)
                x = R.to_device(ci.x, dtype)
                sentinel = float("nan") if out_mode == B.SC_OUT_ZERO_FILL else 7.0
                B.sparse_conv_plan_set_option(layer.plan, B.SC_OPT_MASKED_STORE, 1)
                a = layer.new_output().fill_(sentinel)
                layer.sparse(x, a)
                B.sparse_conv_plan_set_option(layer.plan, B.SC_OPT_MASKED_STORE, 2)
                assert B.sparse_conv_plan_tiles(layer.plan, 0)[2] == -(-spec.m // 64) * -(-spec.c_out // 64)   # every row
                assert B.sparse_conv_plan_kernel(layer.plan, 0) == "tile_masked_store"
                b = layer.new_output().fill_(sentinel)
                layer.sparse(x, b)
                torch.cuda.synchronize()
                assert np.array_equal(R.bits_of(a), R.bits_of(b)), (case, dtype, out_mode)
    # and against the oracle, with the tile left to the plan
    spec = spec_of(8, 192, 7, 7, 32, k=1, p=0, dtype="bf16", sp=0.5)
    ci = W.make_conv_inputs(spec, 1111)
    layer = R.ConvLayer(spec, ci.w, ci.bias, ci.mask)
    B.sparse_conv_plan_set_option(layer.plan, B.SC_OPT_MASKED_STORE, 2)
    y = layer.new_output(fill_nan=True)
    layer.sparse(R.to_device(ci.x, "bf16"), y)
    torch.cuda.synchronize()
    ref, absum = oracle.masked_conv2d(spec, ci.x, ci.w, ci.bias, ci.mask, want_absum=True)
    kept = ci.mask == 1
    assert (rows_view(spec, R.bits_of(y))[~kept] == 0).all()
    assert_close(rows_view(spec, R.to_host_f32(y))[kept], rows_view(spec, ref)[kept], rows_view(spec, absum)[kept], TOL["bf16"])


@pytest.mark.parametrize("case", [
    dict(n=16, cin=512, h=7, w=7, cout=512, sp=0.5),             # deep: K splits are candidates
    dict(n=8, cin=192, h=7, w=7, cout=32, k=1, p=0, sp=0.5),     # tiny pointwise layer: the masked-store variant is one
    dict(n=4, cin=64, h=28, w=28, cout=64, sp=0.5),              # a band-kernel layer
    dict(n=2, cin=96, h=28, w=28, cout=576, k=1, p=0, sp=0.5),   # row-panel kernel
    dict(n=1, cin=3, h=64, w=64, cout=64, k=7, s=2, p=3, sp=0.5),  # row-segment gather: one shape, nothing to choose
])
def test_measured_choice_keeps_the_results(case):
    """sparse_conv_plan_tune replaces the model's choice by the fastest measured one; whatever it picks, both runs match
    the oracle, y holds the sparse run on return, and a new mask returns the sparse run to the model's choice."""
    spec = spec_of(dtype="bf16", **case)
    ci = W.make_conv_inputs(spec, 1120)
    layer = R.ConvLayer(spec, ci.w, ci.bias, ci.mask)
    x = R.to_device(ci.x, "bf16")
    y = layer.new_output(fill_nan=True)
    B.sparse_conv_plan_tune(layer.plan, x, layer.bias, y)
    torch.cuda.synchronize()
    ref, absum = oracle.masked_conv2d(spec, ci.x, ci.w, ci.bias, ci.mask, want_absum=True)
    kept = ci.mask == 1
    assert (rows_view(spec, R.bits_of(y))[~kept] == 0).all()
    assert_close(rows_view(spec, R.to_host_f32(y))[kept], rows_view(spec, ref)[kept], rows_view(spec, absum)[kept], TOL["bf16"])
    yd = layer.new_output(fill_nan=True)
    layer.dense(x, yd)
    torch.cuda.synchronize()
    refd, absd = oracle.masked_conv2d(spec, ci.x, ci.w, ci.bias, np.ones_like(ci.mask), want_absum=True)
    assert_close(rows_view(spec, R.to_host_f32(yd)), rows_view(spec, refd), rows_view(spec, absd), TOL["bf16"])
    # a refreshed mask: the plan still computes the right thing with its new row count
    mask2 = W.gen_mask(spec.m, W.n_keep(0.5, spec.m), 77)
    B.sparse_conv_plan_set_mask(layer.plan, torch.from_numpy(mask2).to("cuda:0"))
    y2 = layer.new_output(fill_nan=True)
    layer.sparse(x, y2)
    torch.cuda.synchronize()
    ref2, abs2 = oracle.masked_conv2d(spec, ci.x, ci.w, ci.bias, mask2, want_absum=True)
    k2 = mask2 == 1
    assert (rows_view(spec, R.bits_of(y2))[~k2] == 0).all()
    assert_close(rows_view(spec, R.to_host_f32(y2))[k2], rows_view(spec, ref2)[k2], rows_view(spec, abs2)[k2], TOL["bf16"])


BAND_CASES = [
    dict(n=3, cin=64, h=20, w=20, cout=64),                         # 3x3, two filter blocks
    dict(n=2, cin=32, h=23, w=17, cout=32, sp=0.3),                 # one filter block, ragged band at the bottom
    dict(n=2, cin=16, h=19, w=31, cout=128, sp=0.6),                # four filter blocks
    dict(n=2, cin=32, h=21, w=21, cout=160, sp=0.5),                # two channel tiles, the second ragged
    dict(n=2, cin=16, h=22, w=18, cout=48, k=3, s=2, p=1, sp=0.4),  # stride 2
    dict(n=1, cin=16, h=24, w=20, cout=32, k=3, p=2, d=2, sp=0.5),  # dilation 2
    dict(n=2, cin=16, h=18, w=26, cout=32, k=5, p=2, sp=0.5),       # 5x5
    dict(n=2, cin=32, h=17, w=15, cout=64, k=3, kw=1, p=1, pw=0, sp=0.5),   # 3x1 window
    dict(n=1, cin=64, h=12, w=12, cout=64, sp=0.95),                # bands with almost no kept rows
]


@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
@pytest.mark.parametrize("mask_mode", ["row", "spatial"])
@pytest.mark.parametrize("case", range(len(BAND_CASES)))
def test_band_kernel(case, mask_mode, dtype, monkeypatch):
    monkeypatch.setenv("SPARSE_CONV_BAND_KERNEL", "single")
    spec = spec_of(dtype=dtype, mask_mode=mask_mode, **BAND_CASES[case])
    eb = 4 if dtype == "f32" else 2
    # the tiled kernel on the same layer (also where the band kernel does not apply)
    check_layer(W.make_conv_inputs(spec, 900 + case), tiles=(64, 64))
    if min(spec.c_out, 128) * spec.k * eb > 96 * 1024:
        return      # filter slab too large for the band kernel at this element size: nothing more to run
    layer = check_layer(W.make_conv_inputs(spec, 900 + case), tiles=(-1, 0))
    assert B.sparse_conv_plan_kernel(layer.plan, 0) == "band"      # really the band kernel


ALT_CASES = [
    dict(n=2, cin=64, h=20, w=20, cout=64),                          # 8 channel groups per pixel, two filter blocks
    dict(n=3, cin=32, h=17, w=19, cout=32, sp=0.3),                  # 4 groups per pixel, one filter block
    dict(n=2, cin=64, h=18, w=18, cout=128, sp=0.4),                 # two channel tiles per band
    dict(n=2, cin=32, h=21, w=21, cout=48, k=3, s=2, p=1, sp=0.5),   # stride 2, ragged channel tile
    dict(n=1, cin=64, h=15, w=13, cout=64, k=3, p=2, d=2, sp=0.6),   # dilation 2
    dict(n=2, cin=32, h=14, w=14, cout=64, sp=0.0),                  # every row kept
    dict(n=1, cin=64, h=12, w=12, cout=64, sp=0.95),                 # bands with almost no kept rows
]


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("mask_mode", ["row", "spatial"])
@pytest.mark.parametrize("case", range(len(ALT_CASES)))
def test_alternating_band_kernel(case, mask_mode, dtype, monkeypatch):
    monkeypatch.setenv("SPARSE_CONV_BAND_KERNEL", "alternating")
    spec = spec_of(dtype=dtype, mask_mode=mask_mode, **ALT_CASES[case])
    layer = check_layer(W.make_conv_inputs(spec, 930 + case), tiles=(-1, 0))
    assert B.sparse_conv_plan_kernel(layer.plan, 0) == "band_alternating"
    assert B.sparse_conv_plan_kernel(layer.plan, 1) == "band_alternating"


@pytest.mark.parametrize("bh,h,w,sp", [(1, 100, 8, 0.5), (1, 40, 12, 0.3), (2, 130, 10, 0.6), (3, 100, 16, 0.5)])
def test_alternating_band_kernel_many_steps(bh, h, w, sp, monkeypatch):
    # more bands than workgroups: every workgroup walks two to four bands, the last step ragged
    monkeypatch.setenv("SPARSE_CONV_BAND_KERNEL", "alternating")
    monkeypatch.setenv("SPARSE_CONV_BAND_HEIGHT", str(bh))
    spec = spec_of(8, 32, h, w, 64, dtype="bf16", sp=sp)
    layer = check_layer(W.make_conv_inputs(spec, 940 + bh + h), tiles=(-1, 0))
    tm, tn, wgs = B.sparse_conv_plan_tiles(layer.plan, 0)
    assert (tm, tn) == (-bh, 64) and wgs == 256 and 8 * ((h + bh - 1) // bh) > 256
    assert B.sparse_conv_plan_kernel(layer.plan, 0) == "band_alternating"


@pytest.mark.parametrize("bh,n,h,w,sp,s", [(7, 3, 23, 20, 0.5, 1), (5, 2, 17, 9, 0.4, 1), (4, 2, 10, 7, 0.6, 1), (3, 1, 3, 5, 0.5, 1),
                                           (7, 40, 56, 16, 0.5, 1), (6, 2, 31, 11, 0.3, 2), (7, 2, 20, 20, 0.0, 1)])
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_alternating_band_kernel_with_split_bands(bh, n, h, w, sp, s, dtype, monkeypatch):
    """Runs of bh output rows cut into two bands of half their pixels: the cut falls inside a row when bh * Wo is
    odd or bh is; the last run of an image may be shorter; 40 images x 8 runs: more bands than workgroups."""
    monkeypatch.setenv("SPARSE_CONV_BAND_KERNEL", "alternating")
    monkeypatch.setenv("SPARSE_CONV_BAND_HEIGHT", f"{bh},split")
    spec = spec_of(n, 64, h, w, 64, dtype=dtype, sp=sp, s=s, mask_mode="spatial" if n == 3 else "row")
    layer = check_layer(W.make_conv_inputs(spec, 960 + bh + h), tiles=(-1, 0), sample_rows=None if n * h * w < 4000 else 400)
    tm, tn, wgs = B.sparse_conv_plan_tiles(layer.plan, 0)
    runs = n * ((spec.ho + bh - 1) // bh)
    assert (tm, tn) == (-bh, 64) and wgs == min(2 * runs, 256)
    assert B.sparse_conv_plan_kernel(layer.plan, 0) == "band_alternating"


def test_tap_kernel_is_the_automatic_choice_when_one_round_of_workgroups_covers_the_layer():
    """The benchmark layer: 256 runs of 7 rows for 256 compute units; sparse and dense runs alike."""
    for sp in (0.5, 0.7, 0.4, 0.25):
        spec = spec_of(32, 64, 56, 56, 64, dtype="bf16", sp=sp)
        layer = R.ConvLayer(spec, *_wbm(spec, 3))
        assert B.sparse_conv_plan_kernel(layer.plan, 0) == "band_tap", sp
        assert B.sparse_conv_plan_kernel(layer.plan, 1) == "band_tap"
        assert B.sparse_conv_plan_tiles(layer.plan, 1) == (-7, 64, 256)


def test_split_bands_of_the_alternating_kernel_when_every_workgroup_gets_one_run(monkeypatch):
    """Without the tap-pipelined kernel: sparse and dense runs decide separately whether to cut their runs of rows."""
    monkeypatch.setenv("SPARSE_CONV_BAND_KERNEL", "no-tap")
    for sp, want in [(0.5, "band_alternating"), (0.7, "band_alternating"), (0.4, "band"), (0.25, "band")]:
        spec = spec_of(32, 64, 56, 56, 64, dtype="bf16", sp=sp)
        layer = R.ConvLayer(spec, *_wbm(spec, 3))
        assert B.sparse_conv_plan_kernel(layer.plan, 0) == want, sp
        assert B.sparse_conv_plan_kernel(layer.plan, 1) == "band_alternating"
        assert B.sparse_conv_plan_tiles(layer.plan, 1) == (-7, 64, 256)


def test_alternating_band_kernel_is_the_automatic_choice_for_long_band_lists(monkeypatch):
    big = spec_of(64, 64, 56, 56, 64, dtype="bf16", sp=0.5)
    layer = R.ConvLayer(big, *_wbm(big, 3))
    assert B.sparse_conv_plan_kernel(layer.plan, 0) == "band_alternating"
    small = spec_of(2, 64, 20, 20, 64, dtype="bf16", sp=0.5)
    layer = R.ConvLayer(small, *_wbm(small, 3))
    assert B.sparse_conv_plan_kernel(layer.plan, 0) == "band_tap"
    monkeypatch.setenv("SPARSE_CONV_BAND_KERNEL", "no-tap")
    layer = R.ConvLayer(small, *_wbm(small, 3))
    assert B.sparse_conv_plan_kernel(layer.plan, 0) == "band"


SPLITK_CASES = [
    dict(n=2, cin=128, h=14, w=14, cout=128),                         # 18 K tiles, 2 x 1 output tiles
    dict(n=1, cin=128, h=20, w=17, cout=256, sp=0.3),                 # two channel tiles, ragged row tile
    dict(n=2, cin=256, h=9, w=9, cout=160, sp=0.6),                   # ragged channel tile, 36 K tiles
    dict(n=1, cin=512, h=7, w=7, cout=512, sp=0.5),                   # the deepest ResNet18 shape: 72 K tiles
    dict(n=2, cin=128, h=15, w=15, cout=128, k=3, s=2, p=1, sp=0.4),  # stride 2
    dict(n=4, cin=1024, h=8, w=8, cout=128, k=1, p=0, sp=0.5),        # pointwise with a long K
]


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("splits", [2, 3, 7])
@pytest.mark.parametrize("case", range(len(SPLITK_CASES)))
def test_split_k_kernel(case, splits, dtype):
    spec = spec_of(dtype=dtype, **SPLITK_CASES[case])
    layer = check_layer(W.make_conv_inputs(spec, 980 + case), split_k=splits)
    assert B.sparse_conv_plan_kernel(layer.plan, 0) == "tile_split_k"
    tm, tn, wgs = B.sparse_conv_plan_tiles(layer.plan, 0)
    tiles = -(-layer.info["kept"] // 64) * -(-spec.c_out // 128)
    assert (tm, tn) == (64, 128) and wgs % tiles == 0 and 2 <= wgs // tiles <= splits


@pytest.mark.parametrize("tile", [(256, 128), (128, 256), (128, 128), (96, 128), (64, 128), (128, 64), (64, 64)])
def test_split_k_every_tile_shape(tile):
    spec = spec_of(2, 256, 12, 12, 160, dtype="bf16", sp=0.4)        # 36 K tiles, ragged rows and channels
    layer = check_layer(W.make_conv_inputs(spec, 989), tiles=tile, split_k=5)
    tm, tn, wgs = B.sparse_conv_plan_tiles(layer.plan, 0)
    assert (tm, tn) == tile and wgs == 5 * -(-layer.info["kept"] // tile[0]) * -(-spec.c_out // tile[1])
    assert B.sparse_conv_plan_kernel(layer.plan, 0) == "tile_split_k"


def test_split_k_on_request_and_never():
    spec = spec_of(64, 512, 7, 7, 512, dtype="bf16", sp=0.5)        # the deepest ResNet18 layers at batch 64
    ci = W.make_conv_inputs(spec, 990)
    layer = check_layer(ci, sample_rows=128)
    # automatic: at most four splits of a tile that has the buffer-load split kernel, priced against the unsplit launches
    if B.sparse_conv_plan_kernel(layer.plan, 0) == "tile_split_k":
        tm, tn, wgs = B.sparse_conv_plan_tiles(layer.plan, 0)
        assert (tm, tn) in ((256, 128), (128, 256), (128, 128), (96, 128), (64, 128))
        assert 2 <= wgs // (-(-layer.info["kept"] // tm) * -(-512 // tn)) <= 4
    B.sparse_conv_plan_set_option(layer.plan, B.SC_OPT_SPLIT_K, 2)
    assert B.sparse_conv_plan_kernel(layer.plan, 0) == "tile_split_k"
    assert B.sparse_conv_plan_tiles(layer.plan, 0) == (64, 128, 2 * 25 * 4)
    B.sparse_conv_plan_set_option(layer.plan, B.SC_OPT_SPLIT_K, 1)
    assert B.sparse_conv_plan_kernel(layer.plan, 0) == "tile_lds_direct"


BUFFER_CASES = [
    # Cin a multiple of 64 and at least three K tiles: the buffer-load form of the tiled kernel
    dict(n=2, cin=64, h=13, w=11, cout=96, k=3, p=1),                        # padded taps on every side
    dict(n=1, cin=128, h=9, w=14, cout=64, k=3, s=2, p=1, sp=0.4),           # stride 2
    dict(n=2, cin=64, h=12, w=12, cout=48, k=3, p=2, d=2, sp=0.6),           # dilation 2
    dict(n=2, cin=64, h=10, w=9, cout=80, k=5, p=2, sp=0.5),                 # 5x5 window: 25 taps
    dict(n=1, cin=64, h=16, w=7, cout=64, k=3, kw=1, p=1, pw=0, sp=0.5),     # 3x1 window
    dict(n=3, cin=256, h=6, w=6, cout=160, k=1, p=0, sp=0.5),                # pointwise, four K tiles, ragged channels
    dict(n=2, cin=192, h=8, w=8, cout=32, k=1, p=0, s=2, sp=0.4),            # strided pointwise, three K tiles
    dict(n=3, cin=64, h=9, w=9, cout=128, k=1, p=0, s=2, sp=0.5),            # one K tile: ring of two
    dict(n=2, cin=128, h=10, w=7, cout=96, k=1, p=0, sp=0.3),                # two K tiles: ring of two
]


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("tile", [(256, 128), (128, 256), (128, 128), (128, 64), (96, 128), (64, 128), (64, 64), (128, 32), (32, 128)])
@pytest.mark.parametrize("case", range(len(BUFFER_CASES)))
def test_buffer_load_tiled_kernel(case, tile, dtype):
    spec = spec_of(dtype=dtype, **BUFFER_CASES[case])
    layer = check_layer(W.make_conv_inputs(spec, 1000 + case), tiles=tile)
    assert B.sparse_conv_plan_kernel(layer.plan, 0) == "tile_lds_direct"
    # (at most two K tiles with the 128 x 128 shape: the buffer-load form has no two-tile ring for it and the
    # global_load_lds form runs in both halves of the comparison below -- the oracle check above is what counts there)
    # the global_load_lds form of the same tile must agree with it (same K order: bitwise)
    ci = W.make_conv_inputs(spec, 1000 + case)
    x = R.to_device(ci.x, spec.dtype)
    a = R.bits_of(layer.sparse(x)).copy()
    B.sparse_conv_plan_set_option(layer.plan, B.SC_OPT_GATHER_PIPELINE, 2)
    assert np.array_equal(R.bits_of(layer.sparse(x)), a)


def test_split_k_repeated_launches_leave_the_counters_clean():
    # the arrival counters are reset by the workgroup that finishes a tile: many launches in a row,
    # sparse and dense interleaved, must all give the first launch's bits
    spec = spec_of(2, 256, 10, 10, 256, dtype="bf16", sp=0.5)
    ci = W.make_conv_inputs(spec, 991)
    layer = R.ConvLayer(spec, ci.w, ci.bias, ci.mask)
    B.sparse_conv_plan_set_option(layer.plan, B.SC_OPT_SPLIT_K, 3)
    assert B.sparse_conv_plan_kernel(layer.plan, 0) == "tile_split_k"
    x = R.to_device(ci.x, spec.dtype)
    first_s = R.bits_of(layer.sparse(x)).copy()
    first_d = R.bits_of(layer.dense(x)).copy()
    for _ in range(20):
        assert np.array_equal(R.bits_of(layer.sparse(x)), first_s)
        assert np.array_equal(R.bits_of(layer.dense(x)), first_d)


PANEL_CASES = [
    dict(n=2, cin=96, h=15, w=15, cout=576, k=1, p=0),                   # two K tiles, nine channel tiles, ragged row tile
    dict(n=3, cin=32, h=14, w=13, cout=192, k=1, p=0, sp=0.3),           # one K tile (half used), three channel tiles
    dict(n=2, cin=128, h=12, w=12, cout=160, k=1, p=0, sp=0.6),          # ragged last channel tile
    dict(n=4, cin=64, h=17, w=17, cout=128, k=1, p=0, s=2, sp=0.5),      # strided pointwise (downsample)
    dict(n=1, cin=16, h=40, w=24, cout=48, k=1, p=0, sp=0.9),            # few kept rows, long zero-fill ranges
    dict(n=2, cin=8, h=11, w=11, cout=64, k=3, p=1, sp=0.5),             # a 3x3 window with K = 72
    dict(n=2, cin=64, h=10, w=10, cout=1024, k=1, p=0, sp=0.0),          # widest bias slice, every row kept
]


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("mask_mode", ["row", "spatial"])
@pytest.mark.parametrize("case", range(len(PANEL_CASES)))
def test_row_panel_kernel(case, mask_mode, dtype):
    spec = spec_of(dtype=dtype, mask_mode=mask_mode, **PANEL_CASES[case])
    layer = check_layer(W.make_conv_inputs(spec, 960 + case), row_panel=2)
    assert B.sparse_conv_plan_kernel(layer.plan, 0) == "tile_row_panel"
    assert B.sparse_conv_plan_kernel(layer.plan, 1) == "tile_row_panel"
    assert B.sparse_conv_plan_tiles(layer.plan, 0) == (128, 64, -(-layer.info["kept"] // 128))


def test_row_panel_kernel_scatter_only_and_switch():
    spec = spec_of(2, 96, 16, 16, 192, k=1, p=0, dtype="bf16", sp=0.5)
    layer = check_layer(W.make_conv_inputs(spec, 969), out_mode=B.SC_OUT_SCATTER_ONLY, row_panel=2)
    assert B.sparse_conv_plan_kernel(layer.plan, 0) == "tile_row_panel"
    B.sparse_conv_plan_set_option(layer.plan, B.SC_OPT_ROW_PANEL, 0)      # too few rows for the automatic choice
    assert B.sparse_conv_plan_kernel(layer.plan, 0) in ("tile_lds_direct", "tile_masked_store")
    big = spec_of(64, 96, 56, 56, 576, k=1, p=0, dtype="bf16", sp=0.5)
    layer = R.ConvLayer(big, *_wbm(big, 3))
    assert B.sparse_conv_plan_kernel(layer.plan, 0) == "tile_row_panel"
    B.sparse_conv_plan_set_option(layer.plan, B.SC_OPT_ROW_PANEL, 1)
    assert B.sparse_conv_plan_kernel(layer.plan, 0) == "tile_lds_direct"


ROWSEG_CASES = [
    # NHWC, Cin * 2 bytes not a multiple of 16, W * Cin a multiple of 8: window-row segments from a padded copy
    dict(n=2, cin=3, h=37, w=40, cout=64, k=7, s=2, p=3),                    # stem-like: 21 entries per window row
    dict(n=2, cin=4, h=15, w=18, cout=32, k=3, p=1, sp=0.3),                 # 12 entries per row, half a group of tail
    dict(n=3, cin=1, h=19, w=32, cout=16, k=5, p=2, sp=0.6),                 # one channel: 5 entries per row
    dict(n=1, cin=2, h=21, w=20, cout=24, k=3, p=2, d=2, dw=1, pw=1, sp=0.5),   # vertical dilation, scalar stores
    dict(n=2, cin=3, h=16, w=24, cout=48, k=3, s=1, p=1, sp=0.4),            # 9 entries per row: two groups
    dict(n=2, cin=6, h=12, w=12, cout=64, k=3, kw=5, p=1, pw=2, sp=0.5),     # 30 entries per row: four groups
    dict(n=1, cin=3, h=14, w=16, cout=64, k=3, p=0, sp=0.0),                 # no padding, every row kept
]


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("mask_mode", ["row", "spatial"])
@pytest.mark.parametrize("case", range(len(ROWSEG_CASES)))
def test_row_segment_gather(case, mask_mode, dtype):
    spec = spec_of(dtype=dtype, mask_mode=mask_mode, **ROWSEG_CASES[case])
    layer = check_layer(W.make_conv_inputs(spec, 1020 + case))
    # (window starts on 4-byte boundaries and 16-channel output groups: the band kernel of these layers serves the
    # automatic launch)
    assert B.sparse_conv_plan_kernel(layer.plan, 0) == ("band_row_segments" if case in (0, 1, 5) else "tile_row_segments")
    for tile in ((64, 64), (128, 32)):
        layer = check_layer(W.make_conv_inputs(spec, 1020 + case), tiles=tile)
        assert B.sparse_conv_plan_kernel(layer.plan, 0) == "tile_row_segments"


def test_row_segment_gather_ignores_non_finite_neighbours():
    # the last 16-byte group of a window row reaches past the window: an infinity there must not
    # turn the (zero-weight) product into NaN
    spec = spec_of(1, 3, 8, 16, 16, k=3, p=1, dtype="bf16", sp=0.0, relu=False)
    ci = W.make_conv_inputs(spec, 1030)
    x = ci.x.copy()
    x[0, 4, 9, :] = np.inf                      # poisons only the windows that contain pixel (4, 9)
    layer = R.ConvLayer(spec, ci.w, ci.bias, ci.mask)
    assert B.sparse_conv_plan_kernel(layer.plan, 0) == "tile_row_segments"
    y = R.to_host_f32(layer.sparse(R.to_device(x, "bf16")))
    touched = np.zeros((8, 16), bool)
    touched[3:6, 8:11] = True
    assert np.isfinite(y[0][~touched]).all()
    assert not np.isfinite(y[0][touched]).all()


STREAM_CASES = [
    dict(n=2, cin=64, h=14, w=14, cout=128),                         # 128 channels: one channel tile
    dict(n=1, cin=128, h=12, w=10, cout=256, sp=0.3),                # two channel tiles, two K tiles per tap
    dict(n=2, cin=64, h=18, w=18, cout=128, k=3, s=2, p=1, sp=0.4),  # stride 2
    dict(n=1, cin=64, h=13, w=15, cout=192, k=3, p=2, d=2, sp=0.5),  # dilation 2, ragged second channel tile
    dict(n=1, cin=256, h=9, w=9, cout=128, sp=0.6),                  # four K tiles per tap
    dict(n=2, cin=64, h=11, w=12, cout=160, k=5, p=2, sp=0.5),       # 5x5 window
]


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("mask_mode", ["row", "spatial"])
@pytest.mark.parametrize("case", range(len(STREAM_CASES)))
def test_streaming_band_kernel(case, mask_mode, dtype):
    spec = spec_of(dtype=dtype, mask_mode=mask_mode, **STREAM_CASES[case])
    layer = check_layer(W.make_conv_inputs(spec, 950 + case), tiles=(-1, 0))
    assert B.sparse_conv_plan_kernel(layer.plan, 0) == "band_stream"


@pytest.mark.parametrize("bh,sp", [(4, 0.5), (7, 0.5), (10, 0.3), (12, 0.1), (12, 0.6)])
def test_streaming_band_kernel_tall_bands(bh, sp, monkeypatch):
    # band heights that put 128 .. 384 rows into one workgroup: 1 .. 3 accumulator blocks per wavefront
    monkeypatch.setenv("SPARSE_CONV_BAND_HEIGHT", str(bh))
    spec = spec_of(2, 64, 32, 32, 128, dtype="bf16", sp=sp)
    layer = check_layer(W.make_conv_inputs(spec, 970 + bh), tiles=(-1, 0))
    assert B.sparse_conv_plan_tiles(layer.plan, 0)[0] == -bh


def test_band_kernel_scatter_only_and_empty():
    spec = spec_of(2, 32, 16, 16, 64, dtype="bf16", sp=0.5)
    ci = W.make_conv_inputs(spec, 41)
    check_layer(ci, tiles=(-1, 0), out_mode=B.SC_OUT_SCATTER_ONLY)
    ci.mask[:] = 0
    ci.mask[100] = 1
    check_layer(ci, tiles=(-1, 0), check_count=False)


def _wbm(spec, seed):
    ci = W.make_conv_inputs(spec, seed, x=np.zeros(1, np.float32))
    return ci.w, ci.bias, ci.mask


@pytest.mark.parametrize("layout", ["nhwc", "nchw"])
def test_spatial_mask_shared_by_the_batch(layout):
    spec = spec_of(3, 16, 13, 17, 32, dtype="bf16", layout=layout, sp=0.4, mask_mode="spatial")
    ci = W.make_conv_inputs(spec, 11)
    assert ci.mask.size == spec.ho * spec.wo
    check_layer(ci)


@pytest.mark.parametrize("layout", ["nhwc", "nchw"])
def test_scatter_only_leaves_dropped_rows_alone(layout):
    spec = spec_of(2, 16, 15, 15, 32, dtype="bf16", layout=layout, sp=0.5)
    check_layer(W.make_conv_inputs(spec, 13), out_mode=B.SC_OUT_SCATTER_ONLY)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_all_rows_dropped_and_all_rows_kept(dtype):
    spec = spec_of(2, 16, 9, 9, 24, dtype=dtype, sp=0.5)
    ci = W.make_conv_inputs(spec, 17)
    ci.mask[:] = 0
    check_layer(ci, check_count=False)
    ci.mask[:] = 1
    check_layer(ci, check_count=False)
    ci.mask[:] = 0
    ci.mask[-1] = 1                                    # a single kept row, the last one
    check_layer(ci, check_count=False)
    ci.mask[:] = 1
    ci.mask[0] = 0
    check_layer(ci, check_count=False)


def test_any_nonzero_mask_byte_keeps_the_row():
    spec = spec_of(1, 16, 8, 8, 16, dtype="bf16", sp=0.5)
    ci = W.make_conv_inputs(spec, 19)
    odd = ci.mask.copy()
    odd[odd == 1] = np.random.default_rng(0).integers(1, 256, int(odd.sum())).astype(np.uint8)
    layer = R.ConvLayer(spec, ci.w, ci.bias, odd)
    assert np.array_equal(B.plan_row_idx(layer.plan).cpu().numpy(), oracle.compact_rows(ci.mask))


def test_mask_count_must_match_the_sparsity_ratio():
    spec = spec_of(1, 16, 8, 8, 16, dtype="bf16", sp=0.5)
    ci = W.make_conv_inputs(spec, 23)
    bad = ci.mask.copy()
    bad[np.flatnonzero(bad)[0]] = 0
    with pytest.raises(B.ScError) as e:
        R.ConvLayer(spec, ci.w, ci.bias, bad)
    assert e.value.status == B.SC_ERR_MASK_COUNT
    R.ConvLayer(spec, ci.w, ci.bias, bad, check_count=False)      # a negative ratio disables the check


def test_mask_count_at_a_half_within_the_float_rounding_of_the_ratio():
    """(1 - 0.9) * 135 is 13.5 up to the rounding of 0.9: in double the count is 13, from the descriptor's float 14.  A
    mask with either count is the one the caller's ratio demands; 12 and 15 are not."""
    spec = spec_of(1, 64, 7, 13, 16, k=3, p=3, d=2, dtype="bf16", sp=0.9, mask_mode="spatial")
    assert spec.ho * spec.wo == 135
    ci = W.make_conv_inputs(spec, 24)
    assert int(ci.mask.sum()) == 13
    for kept, ok in ((12, False), (13, True), (14, True), (15, False)):
        mask = np.zeros(135, np.uint8)
        mask[:kept] = 1
        if ok:
            R.ConvLayer(spec, ci.w, ci.bias, mask)
        else:
            with pytest.raises(B.ScError) as e:
                R.ConvLayer(spec, ci.w, ci.bias, mask)
            assert e.value.status == B.SC_ERR_MASK_COUNT


@pytest.mark.parametrize("m", [1, 63, 64, 65, 1023, 1024, 1025, 4096, 100352, 802816])
def test_compaction_sizes(m):
    # a0 on its own: m one-pixel "images" of a pointwise layer; the row list must equal the oracle's
    spec = W.ConvSpec("cmp", n=m, c_in=8, h=1, w=1, c_out=16, kh=1, kw=1, pad_h=0, pad_w=0, dtype="bf16", sparsity=0.37)
    mask = W.gen_mask(m, W.n_keep(0.37, m), 3 + m)
    w = np.zeros(spec.w_shape(), np.float32)
    layer = R.ConvLayer(spec, w, np.zeros(16, np.float32), mask)
    want = oracle.compact_rows(mask)
    assert layer.info["kept"] == want.size == oracle.kept_count(0.37, m)
    assert np.array_equal(B.plan_row_idx(layer.plan).cpu().numpy(), want)


@pytest.mark.parametrize("s", W.C2_SPARSITIES)
def test_config2_full_size(s):
    spec = W.config2(s)
    ci = W.make_conv_inputs(spec, W.base_seed(2))
    assert ci.keep == {0.0: 100352, 0.25: 75264, 0.5: 50176, 0.7: 30106}[s]
    check_layer(ci)


@pytest.mark.parametrize("idx", range(16))
def test_config4_pointwise(idx):
    spec = W.config4()[idx]
    check_layer(W.make_conv_inputs(spec, W.base_seed(4)))


def test_glue_ops_match_oracle():
    rng = np.random.default_rng(8)
    # 24 channels: eight per thread for the 16-bit types; 5 channels: the element-wise kernels
    for dtype, shape in [(d, sh) for d in ("bf16", "f16", "f32") for sh in ((3, 13, 10, 24), (2, 9, 11, 5))]:
        x = W.quantize(rng.standard_normal(shape).astype(np.float32), dtype)
        y = B.sc_maxpool2d_nhwc(R.to_device(x, dtype), 3, 2, 1)
        assert np.array_equal(R.to_host_f32(y), oracle.maxpool2d_nhwc(x, 3, 2, 1))
        b = W.quantize(rng.standard_normal(x.shape).astype(np.float32), dtype)
        z = B.sc_add_relu(R.to_device(x, dtype), R.to_device(b, dtype))
        assert np.array_equal(R.to_host_f32(z), oracle.round_storage(oracle.add_relu(x, b), dtype))
        z = B.sc_add(R.to_device(x, dtype), R.to_device(b, dtype))
        want = oracle.round_storage((x.astype(np.float64) + b).astype(np.float32), dtype)
        assert np.array_equal(R.to_host_f32(z), want)


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("k,s,p", [(3, 2, 1), (3, 1, 1), (3, 2, 0), (3, 3, 1), (2, 2, 0), (5, 2, 2)])
def test_maxpool_windows(k, s, p, dtype):
    # the 3x3 window has a kernel of its own (nine unconditional loads); other windows walk their taps
    rng = np.random.default_rng(80 + k + s + p)
    for shape in ((2, 17, 21, 64), (1, 8, 8, 8), (3, 5, 30, 40)):
        x = W.quantize(rng.standard_normal(shape).astype(np.float32), dtype)
        x[0, 0, 0, :] = -np.inf
        y = B.sc_maxpool2d_nhwc(R.to_device(x, dtype), k, s, p)
        assert np.array_equal(R.to_host_f32(y), oracle.maxpool2d_nhwc(x, k, s, p))


def _run_network_both(ops, bs, batch_note=""):
    """Run an op list through the HIP path and through the oracle from the same synthetic input."""
    params = {}

    def layer_inputs(spec):
        if spec.name not in params:
            ci = W.make_conv_inputs(spec, bs, x=np.zeros(1, np.float32))
            params[spec.name] = (ci.w, ci.bias, ci.mask)
        return params[spec.name]

    dtype = W.conv_specs(ops)[0].dtype
    host = {"input": W.gen_activations(W.network_input_shape(ops), bs, dtype)}
    for op in ops:
        if op.kind == "conv" and op.src.startswith("synthetic:"):
            host[op.src] = W.gen_activations(op.spec.x_shape(), bs + 500 + op.spec.layer_index, dtype)
    layers = {s.name: R.ConvLayer(s, *layer_inputs(s)) for s in W.conv_specs(ops)}
    dev = R.run_network(ops, {k: R.to_device(v, dtype) for k, v in host.items()}, layers)
    torch.cuda.synchronize()
    absums = {}
    ref = oracle.run_network(ops, host, layer_inputs, absums=absums)
    return dev, ref, params, absums


def test_config3_resnet18_stack_small_batch():
    ops = W.config3(batch=4)
    dev, ref, params, absums = _run_network_both(ops, W.base_seed(3))
    compare_network(ops, dev, ref, params, TOL["bf16"], absums)


@pytest.mark.timeout(600)
def test_config3_resnet18_stack_full_batch():
    """The whole configuration: batch 64 at 224 x 224, every element of every tensor of the chain against the oracle."""
    ops = W.config3(batch=64)
    dev, ref, params, absums = _run_network_both(ops, W.base_seed(3))
    compare_network(ops, dev, ref, params, TOL["bf16"], absums)


def test_config3_resnet18_stack_dense_downsample_variant():
    ops = W.config3(batch=2, sparse_downsample=False)
    dev, ref, params, absums = _run_network_both(ops, W.base_seed(3))
    compare_network(ops, dev, ref, params, TOL["bf16"], absums)


def test_config5_detector_stack():
    ops = W.config5(batch=16)
    dev, ref, params, absums = _run_network_both(ops, W.base_seed(5))
    compare_network(ops, dev, ref, params, TOL["bf16"], absums)


def test_fixed_buffer_runner_and_graph_replay_match_the_eager_chain():
    """The same op list through preallocated buffers, call by call and as a HIP graph replayed several
    times with eager work in between: every pass must reproduce the eager chain bit for bit."""
    ops = W.config3(batch=2)
    bs = W.base_seed(3)
    dtype = "bf16"
    layers = {}
    for s in W.conv_specs(ops):
        ci = W.make_conv_inputs(s, bs, x=np.zeros(1, np.float32))
        layers[s.name] = R.ConvLayer(s, ci.w, ci.bias, ci.mask)
    x = R.to_device(W.gen_activations(W.network_input_shape(ops), bs, dtype), dtype)
    eager = R.run_network(ops, {"input": x}, layers)
    want = {op.out: R.bits_of(eager[op.out]).copy() for op in ops}
    net = R.NetworkRunner(ops, {"input": x}, layers)

    def poison_and_check(run):
        for op in ops:
            net.tensors[op.out].fill_(float("nan"))
        run()
        torch.cuda.synchronize()
        for op in ops:
            assert np.array_equal(R.bits_of(net.tensors[op.out]), want[op.out]), op.out

    poison_and_check(net.run)
    graph = net.capture()
    for _ in range(3):
        poison_and_check(graph.replay)
        scratch = torch.randn(1 << 16, device="cuda:0").sum().item()   # unrelated eager work and a sync between replays
        assert np.isfinite(scratch)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("index", range(20))
def test_config3_full_batch_every_row(index):
    """Every ResNet18 layer at batch 64 (the full configuration), each on synthetic input of its own shape, every row of
    the sparse and of the dense run through the oracle."""
    spec = W.conv_specs(W.config3(batch=64))[index]
    ci = W.make_conv_inputs(spec, W.base_seed(3))
    check_layer(ci)
    torch.cuda.empty_cache()


@pytest.mark.parametrize("multiple", [8, 16])
def test_pruned_resnet18_with_padded_channels_matches_the_unpadded_oracle(multiple):
    """Channel counts that are no multiple of 8 (a structurally pruned model): the stack runs with every
    tensor padded to 16-byte channel groups -- zero filters, so the extra channels stay exactly zero --
    and must reproduce the oracle's run of the original shapes."""
    ops = W.pruned_resnet18(batch=2, sparsity=0.3)
    pops = W.pad_channels(ops, multiple)
    assert [s.c_out for s in W.conv_specs(ops)][:2] == [51, 51] and W.conv_specs(pops)[1].c_in == (56 if multiple == 8 else 64)
    bs = W.base_seed(3)
    params, layers = {}, {}
    for spec, pspec in zip(W.conv_specs(ops), W.conv_specs(pops)):
        ci = W.make_conv_inputs(spec, bs, x=np.zeros(1, np.float32))
        params[spec.name] = (ci.w, ci.bias, ci.mask)
        wp, bp = R.pad_conv_params(spec, pspec, ci.w, ci.bias)
        layers[spec.name] = R.ConvLayer(pspec, wp, bp, ci.mask)
        assert "elements" not in B.sparse_conv_plan_kernel(layers[spec.name].plan, 0) or spec.name == "stem"
    dtype = "bf16"
    host = {"input": W.gen_activations(W.network_input_shape(ops), bs, dtype)}
    dev = R.run_network(pops, {k: R.to_device(v, dtype) for k, v in host.items()}, layers)
    torch.cuda.synchronize()
    ref = oracle.run_network(ops, host, lambda spec: params[spec.name])
    trimmed = {}
    for op in ops:
        c = ref[op.out].shape[-1]
        full = dev[op.out]
        assert (R.bits_of(full)[..., c:] == 0).all(), f"{op.out}: padding channels must stay zero"
        trimmed[op.out] = full[..., :c].contiguous()
    compare_network(ops, trimmed, ref, params, TOL["bf16"])
