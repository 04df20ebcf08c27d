"""Slab form of the tiled kernel (deep 3x3 layers: the input pixels under a tile's kept rows stay in LDS per chunk of 32
input channels and are read once per window tap) against the oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import oracle
from paper_2309_06626_amd import binding as B
from paper_2309_06626_amd import runtime as R
from tests.parity import TOL, assert_close, check_layer, row_mask, rows_view

pytestmark = pytest.mark.gpu


def spec_of(n, cin, h, w, cout, p=1, dtype="bf16", bias=True, relu=True, sp=0.5, mask_mode="row", name="slab", pw=None):
    return W.ConvSpec(name, n=n, c_in=cin, h=h, w=w, c_out=cout, kh=3, kw=3, stride_h=1, stride_w=1, pad_h=p,
                      pad_w=p if pw is None else pw, dil_h=1, dil_w=1, dtype=dtype, layout="nhwc", has_bias=bias, relu=relu,
                      sparsity=sp, mask_mode=mask_mode)


SHAPES = {
    "20x20_64_128": dict(n=2, cin=64, h=20, w=20, cout=128),              # two chunks, one channel tile
    "14x14_128_256": dict(n=3, cin=128, h=14, w=14, cout=256),            # tiles that span several images
    "7x7_96_128": dict(n=12, cin=96, h=7, w=7, cout=128),                 # three chunks; many images per tile
    "9x13_32_96": dict(n=2, cin=32, h=9, w=13, cout=96),                  # one chunk; channel tile partly beyond Cout
    "12x10_64_320_nopad": dict(n=2, cin=64, h=12, w=10, cout=320, p=0),   # no padding; last channel tile half used
    "8x8_64_128_pad2": dict(n=3, cin=64, h=8, w=8, cout=128, p=2),        # output larger than the input
    "10x16_64_144_pads": dict(n=2, cin=64, h=10, w=16, cout=144, p=1, pw=0),
    "28x28_32_128": dict(n=2, cin=32, h=28, w=28, cout=128),              # several row tiles per image
}


def slab_fits(spec, mask, bm):
    """Whether the widest slab of a bm-row tile fits its LDS buffer (40 KB: 64 bytes per pixel of the zero-padded rows
    between the window of the tile's first kept row and that of its last) -- recomputed here from the kept rows."""
    rows = oracle.compact_rows(row_mask(spec, mask))
    if rows.size == 0:
        return False
    hp, wp = spec.h + 2 * spec.pad_h, spec.w + 2 * spec.pad_w
    vrow = (rows // (spec.ho * spec.wo)) * hp + (rows % (spec.ho * spec.wo)) // spec.wo
    first = vrow[::bm]
    last = vrow[np.minimum(np.arange(0, rows.size, bm) + bm, rows.size) - 1]
    span = int((last + 3 - first).max())
    round_bytes = (512 if bm == 256 else 256) * 16
    return -(-span * wp * 64 // round_bytes) * round_bytes <= 40960


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("bm", [128, 256])
@pytest.mark.parametrize("shape", list(SHAPES))
def test_slab_kernel_matches_the_oracle(shape, bm, dtype):
    spec = spec_of(dtype=dtype, **SHAPES[shape])
    ci = W.make_conv_inputs(spec, 2000 + len(shape))
    layer = check_layer(ci, options={B.SC_OPT_SLAB: bm})
    assert (B.sparse_conv_plan_kernel(layer.plan, 0) == "tile_slab") == slab_fits(spec, ci.mask, bm)
    assert (B.sparse_conv_plan_kernel(layer.plan, 1) == "tile_slab") == slab_fits(spec, np.ones_like(ci.mask), bm)
    if slab_fits(spec, ci.mask, bm):
        assert B.sparse_conv_plan_tiles(layer.plan, 0)[:2] == (bm, 128)


@pytest.mark.parametrize("sp,mask_mode", [(0.0, "row"), (0.3, "row"), (0.7, "row"), (0.5, "spatial"), (0.95, "row")])
@pytest.mark.parametrize("bm", [128, 256])
def test_slab_kernel_mask_densities(bm, sp, mask_mode):
    # sparse masks widen the slab of a tile (its kept rows lie further apart): where it no longer fits, another kernel runs
    spec = spec_of(4, 64, 14, 14, 128, sp=sp, mask_mode=mask_mode)
    ci = W.make_conv_inputs(spec, 2100 + bm)
    layer = check_layer(ci, options={B.SC_OPT_SLAB: bm})
    assert (B.sparse_conv_plan_kernel(layer.plan, 0) == "tile_slab") == slab_fits(spec, ci.mask, bm)
    assert slab_fits(spec, ci.mask, 128) == (sp < 0.9)


@pytest.mark.parametrize("out_mode", [B.SC_OUT_ZERO_FILL, B.SC_OUT_SCATTER_ONLY])
@pytest.mark.parametrize("splits", [2, 3, 5])
@pytest.mark.parametrize("bm", [128, 256])
def test_slab_kernel_with_split_chunks(bm, splits, out_mode):
    spec = spec_of(3, 256, 10, 10, 256, sp=0.4)                      # eight chunks; K tiles enough for the split workspace
    ci = W.make_conv_inputs(spec, 2200 + splits)
    layer = check_layer(ci, out_mode=out_mode, split_k=splits, options={B.SC_OPT_SLAB: bm})
    assert slab_fits(spec, ci.mask, bm) and B.sparse_conv_plan_kernel(layer.plan, 0) == "tile_slab"
    tiles = -(-layer.info["kept"] // bm) * 2
    assert B.sparse_conv_plan_tiles(layer.plan, 0)[2] == tiles * splits
    # the arrival counters are left at zero: repeated launches, sparse and dense interleaved, give the same bits
    x = R.to_device(ci.x, spec.dtype)
    y = layer.new_output().fill_(3.0)                 # (scatter-only runs leave the dropped rows as they find them)
    first_s, first_d = R.bits_of(layer.sparse(x, y)).copy(), R.bits_of(layer.dense(x)).copy()
    for _ in range(5):
        assert np.array_equal(R.bits_of(layer.sparse(x, y.fill_(3.0))), first_s)
        assert np.array_equal(R.bits_of(layer.dense(x)), first_d)


def test_slab_kernel_edge_masks():
    spec = spec_of(8, 64, 12, 12, 128, sp=0.5)
    ci = W.make_conv_inputs(spec, 2300)
    for name in ("none", "first", "last", "ends", "all"):
        ci.mask[:] = 1 if name == "all" else 0
        if name in ("first", "ends"):
            ci.mask[0] = 1
        if name in ("last", "ends"):
            ci.mask[-1] = 1
        layer = check_layer(ci, options={B.SC_OPT_SLAB: 2}, check_count=False)
        # "ends": the first and the last row of the tensor in one tile -- a slab of every virtual row does not fit
        assert (B.sparse_conv_plan_kernel(layer.plan, 0) == "tile_slab") == (name in ("first", "last", "all")), name
        assert (slab_fits(spec, ci.mask, 128) or slab_fits(spec, ci.mask, 256)) == (name in ("first", "last", "all")), name


def test_slab_kernel_agrees_with_the_tiled_kernel_on_a_deep_layer():
    spec = spec_of(8, 512, 7, 7, 512, sp=0.5)
    ci = W.make_conv_inputs(spec, 2400)
    layer = check_layer(ci, options={B.SC_OPT_SLAB: 128}, sample_rows=64)
    assert B.sparse_conv_plan_kernel(layer.plan, 0) == "tile_slab"
    x = R.to_device(ci.x, spec.dtype)
    a = R.to_host_f32(layer.sparse(x))
    B.sparse_conv_plan_set_option(layer.plan, B.SC_OPT_SLAB, 1)
    assert B.sparse_conv_plan_kernel(layer.plan, 0) != "tile_slab"
    b = R.to_host_f32(layer.sparse(x))
    # two orders of the same K sum, each rounded once to bf16
    assert np.abs(a - b).max() <= 2 * TOL["bf16"] * max(np.abs(b).max(), 1e-30)


@pytest.mark.parametrize("post_relu", [False, True])
@pytest.mark.parametrize("bm,splits", [(128, 0), (256, 2)])
def test_slab_kernel_with_a_fused_shortcut_and_with_compact_output(bm, splits, post_relu):
    spec = spec_of(3, 256, 12, 12, 256, sp=0.4, relu=False)
    ci = W.make_conv_inputs(spec, 2500 + bm)
    layer = R.ConvLayer(spec, ci.w, ci.bias, ci.mask)
    B.sparse_conv_plan_set_option(layer.plan, B.SC_OPT_SLAB, bm)
    B.sparse_conv_plan_set_option(layer.plan, B.SC_OPT_SPLIT_K, splits)
    assert B.sparse_conv_plan_kernel(layer.plan, 0) == "tile_slab" == B.sparse_conv_plan_fused_kernel(layer.plan, 0)
    rm = row_mask(spec, ci.mask)
    kept = rm == 1
    tol = TOL[spec.dtype]
    rng = np.random.default_rng(2501)
    res = W.quantize(rng.standard_normal(spec.y_shape()).astype(np.float32), spec.dtype)
    x = R.to_device(ci.x, spec.dtype)
    _, absum = oracle.masked_conv2d(spec, ci.x, ci.w, ci.bias, ci.mask, want_absum=True)
    bound = rows_view(spec, absum) + np.abs(rows_view(spec, res))
    # y = post(conv + bias + shortcut); dropped rows of the dense map receive post(shortcut)
    ref = oracle.masked_conv2d_residual(spec, ci.x, ci.w, ci.bias, ci.mask, res, post_relu)
    y = layer.new_output().fill_(float("nan"))
    B.sparse_conv_run_residual(layer.plan, x, layer.bias, R.to_device(res, spec.dtype), y, post_relu)
    torch.cuda.synchronize()
    assert_close(rows_view(spec, R.to_host_f32(y)), rows_view(spec, ref), bound, tol, "fused shortcut")
    # the kept rows only: [kept x Cout], and nothing behind them
    refc = oracle.masked_conv2d_residual(spec, ci.x, ci.w, ci.bias, ci.mask, rows_view(spec, res)[kept], post_relu, y_compact=True)
    yc = torch.full((int(kept.sum()) + 1, spec.c_out), float("nan"), dtype=B.TORCH_DTYPE[spec.dtype], device="cuda:0")
    B.sparse_conv_run_residual(layer.plan, x, layer.bias, R.to_device(np.ascontiguousarray(rows_view(spec, res)[kept]), spec.dtype),
                               yc[:-1], post_relu, B.SC_ROWS_DENSE, B.SC_ROWS_COMPACT)
    torch.cuda.synchronize()
    assert np.isnan(R.to_host_f32(yc[-1:])).all()
    assert_close(R.to_host_f32(yc[:-1]), refc, bound[kept], tol, "compact output, fused shortcut")


def test_tuned_choice_on_a_layer_the_slab_kernel_serves():
    # sparse_conv_plan_tune times the slab form beside the tiled candidates; whichever wins must match the oracle
    spec = spec_of(16, 128, 28, 28, 128, sp=0.5)
    ci = W.make_conv_inputs(spec, 2600)
    layer = R.ConvLayer(spec, ci.w, ci.bias, ci.mask)
    x, y = R.to_device(ci.x, spec.dtype), layer.new_output()
    B.sparse_conv_plan_tune(layer.plan, x, layer.bias, y)
    rows = np.unique(np.random.default_rng(5).integers(0, spec.m, 300)).astype(np.int64)
    kept = row_mask(spec, ci.mask)[rows] == 1
    for dense in (False, True):
        out = (layer.dense if dense else layer.sparse)(x, layer.new_output().fill_(float("nan")))
        torch.cuda.synchronize()
        mask = np.ones_like(ci.mask) if dense else ci.mask
        ref, absum = oracle.masked_conv2d_rows(spec, ci.x, ci.w, ci.bias, mask, rows, want_absum=True)
        sel = np.ones_like(kept) if dense else kept
        assert_close(rows_view(spec, R.to_host_f32(out))[rows][sel], ref[sel], absum[sel], TOL[spec.dtype], f"tuned, dense={dense}")
    assert B.sparse_conv_plan_kernel(layer.plan, 1) in ("tile_slab", "tile_lds_direct", "tile_split_k")
