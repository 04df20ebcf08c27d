"""Band kernel of small-channel layers (row-segment K order, window rows read from a zero-margined slab in LDS)
against the oracle: paper Sec. 3.2 (lower kept windows only, dense product, results back between zeros)."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import oracle
from paper_2309_06626_amd import binding as B
from paper_2309_06626_amd import runtime as R
from tests.parity import TOL, assert_close, check_layer, row_mask, rows_view

pytestmark = pytest.mark.gpu


def spec_of(n, cin, h, w, cout, k=3, s=1, p=1, d=1, dtype="bf16", bias=True, relu=True, sp=0.5, mask_mode="row", kw=None,
            sw=None, pw=None, dw=None, name="rowband"):
    return W.ConvSpec(name, n=n, c_in=cin, h=h, w=w, c_out=cout, kh=k, kw=k if kw is None else kw, stride_h=s,
                      stride_w=s if sw is None else sw, pad_h=p, pad_w=p if pw is None else pw, dil_h=d,
                      dil_w=d if dw is None else dw, dtype=dtype, layout="nhwc", has_bias=bias, relu=relu, sparsity=sp,
                      mask_mode=mask_mode)


CASES = [
    dict(n=2, cin=3, h=37, w=40, cout=64, k=7, s=2, p=3),                      # stem-like: three groups per window row, tail 5
    dict(n=2, cin=4, h=15, w=18, cout=32, k=3, p=1, sp=0.3),                   # half a group of tail, 32 of 64 channels
    dict(n=2, cin=6, h=12, w=12, cout=64, k=3, kw=5, p=1, pw=2, sp=0.5),       # four groups per window row
    dict(n=1, cin=3, h=30, w=48, cout=128, k=5, s=2, p=2, sp=0.4),             # two channel tiles
    dict(n=2, cin=2, h=21, w=20, cout=80, k=3, s=2, p=1, sp=0.5),              # second channel tile of 16 channels
    dict(n=1, cin=4, h=23, w=16, cout=16, k=3, p=2, d=2, dw=1, pw=1, sp=0.5),  # vertical dilation
    dict(n=2, cin=3, h=20, w=32, cout=48, k=3, s=2, sw=4, p=1, sp=0.6),        # strides differ
    dict(n=1, cin=3, h=14, w=16, cout=64, k=3, s=2, p=0, sp=0.0),              # no padding, every row kept
    dict(n=3, cin=1, h=19, w=32, cout=32, k=5, s=2, p=2, sp=0.7),              # one channel
    dict(n=1, cin=3, h=64, w=224, cout=64, k=7, s=2, p=3, sp=0.5),             # full stem width: 112 columns
    dict(n=1, cin=4, h=8, w=200, cout=16, k=8, kw=1, s=1, p=0, sp=0.5),        # eight window rows of one group
]


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("mask_mode", ["row", "spatial"])
@pytest.mark.parametrize("case", range(len(CASES)))
def test_band_row_segments(case, mask_mode, dtype):
    spec = spec_of(dtype=dtype, mask_mode=mask_mode, **CASES[case])
    layer = check_layer(W.make_conv_inputs(spec, 1400 + case))
    assert B.sparse_conv_plan_kernel(layer.plan, 0) == "band_row_segments"
    assert B.sparse_conv_plan_kernel(layer.plan, 1) == "band_row_segments"


@pytest.mark.parametrize("bh", [1, 2, 3, 5])
@pytest.mark.parametrize("sp", [0.1, 0.5, 0.9])
def test_band_heights_and_block_shapes(bh, sp, monkeypatch):
    # 1 .. 5 output rows of 96 columns per workgroup: up to 480 rows, one to four blocks per wavefront
    monkeypatch.setenv("SPARSE_CONV_BAND_HEIGHT", str(bh))
    spec = spec_of(2, 3, 23, 192, 64, k=7, s=2, p=3, dtype="bf16", sp=sp)
    layer = check_layer(W.make_conv_inputs(spec, 1440 + bh))
    assert B.sparse_conv_plan_kernel(layer.plan, 0) == "band_row_segments"
    assert B.sparse_conv_plan_tiles(layer.plan, 0)[0] == -bh


def test_large_slabs(monkeypatch):
    # more 16-byte pieces than one pass of the workgroup stages (19 rows of 127 pieces), and more than 128 slab rows
    monkeypatch.setenv("SPARSE_CONV_BAND_HEIGHT", "3")
    spec = spec_of(1, 6, 40, 168, 32, k=7, kw=3, s=3, sw=1, p=2, pw=1, d=2, dw=1, dtype="bf16", sp=0.5)
    layer = check_layer(W.make_conv_inputs(spec, 1451))
    assert B.sparse_conv_plan_kernel(layer.plan, 0) == "band_row_segments" and B.sparse_conv_plan_tiles(layer.plan, 0)[0] == -3
    monkeypatch.setenv("SPARSE_CONV_BAND_HEIGHT", "1")
    spec = spec_of(2, 1, 150, 8, 16, k=8, kw=3, s=1, sw=2, p=3, pw=1, d=19, dw=1, dtype="f16", sp=0.4)
    layer = check_layer(W.make_conv_inputs(spec, 1452))
    assert B.sparse_conv_plan_kernel(layer.plan, 0) == "band_row_segments"


def test_scatter_only_empty_and_single_row():
    spec = spec_of(2, 3, 18, 24, 64, k=7, s=2, p=3, dtype="bf16", sp=0.5)
    ci = W.make_conv_inputs(spec, 1460)
    layer = check_layer(ci, out_mode=B.SC_OUT_SCATTER_ONLY)
    assert B.sparse_conv_plan_kernel(layer.plan, 0) == "band_row_segments"
    ci.mask[:] = 0
    check_layer(ci, check_count=False)
    ci.mask[77] = 1
    check_layer(ci, check_count=False)


def test_non_finite_neighbours_stay_out():
    # the last 16-byte group of a window row reaches one pixel past the window: an infinity there must not meet the
    # zero filter entries of the padding
    spec = spec_of(1, 4, 8, 16, 16, k=3, p=1, dtype="bf16", sp=0.0, relu=False)
    ci = W.make_conv_inputs(spec, 1470)
    x = ci.x.copy()
    x[0, 4, 9, :] = np.inf                      # poisons only the windows that contain pixel (4, 9)
    layer = R.ConvLayer(spec, ci.w, ci.bias, ci.mask)
    assert B.sparse_conv_plan_kernel(layer.plan, 0) == "band_row_segments"
    y = R.to_host_f32(layer.sparse(R.to_device(x, "bf16")))
    touched = np.zeros((8, 16), bool)
    touched[3:6, 8:11] = True
    assert np.isfinite(y[0][~touched]).all()
    assert not np.isfinite(y[0][touched]).all()


def test_forced_tiles_take_the_tiled_kernel():
    spec = spec_of(2, 3, 37, 40, 64, k=7, s=2, p=3, dtype="bf16")
    for tile in ((64, 64), (128, 32)):
        layer = check_layer(W.make_conv_inputs(spec, 1480), tiles=tile)
        assert B.sparse_conv_plan_kernel(layer.plan, 0) == "tile_row_segments"


def test_tuned_plan_keeps_the_faster_kernel():
    # sparse_conv_plan_tune times the tiled row-segment kernel beside the band; whichever wins must match the oracle
    spec = spec_of(8, 3, 64, 64, 64, k=7, s=2, p=3, dtype="bf16")
    ci = W.make_conv_inputs(spec, 1490)
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
        assert B.sparse_conv_plan_kernel(layer.plan, int(dense)) in ("band_row_segments", "tile_row_segments")


@pytest.mark.parametrize("seed", [11, 23])
def test_random_small_channel_layers(seed):
    """Seeded random window shapes, strides, paddings, dilations, channel counts and band heights of the layers this kernel takes."""
    import os
    import random
    rnd = random.Random(seed)
    done = 0
    while done < 30:
        cin = rnd.choice([1, 2, 3, 3, 4, 6])
        kh, kw = rnd.randint(1, 8), rnd.randint(1, 7)
        sw = rnd.choice([1, 2, 2, 4]) if cin % 2 else rnd.choice([1, 1, 2, 3])
        sh = rnd.choice([1, 2, 2, 3])
        dh = rnd.choice([1, 1, 2])
        gpw = (kw * cin + 7) // 8
        w = rnd.randint(max(kw, 4), 70)
        if (sw * cin) % 2 or kh * kw == 1 or kh * gpw > 24 or (w * cin) % 8:
            continue
        ph, pw = rnd.randint(0, (kh - 1) * dh), rnd.randint(0, kw - 1)
        h = rnd.randint(max((kh - 1) * dh + 1 - 2 * ph, 3), 40)
        cout = 16 * rnd.randint(1, 9)
        spec = spec_of(rnd.randint(1, 4), cin, h, w, cout, k=kh, kw=kw, s=sh, sw=sw, p=ph, pw=pw, d=dh, dw=1,
                       dtype=rnd.choice(["bf16", "f16"]), sp=rnd.choice([0.0, 0.3, 0.5, 0.8, 0.97]),
                       mask_mode=rnd.choice(["row", "spatial"]), relu=rnd.choice([True, False]), bias=rnd.choice([True, False]))
        bh = rnd.choice([0, 0, 1, 2, 3])
        if bh and bh * spec.wo <= 512:
            os.environ["SPARSE_CONV_BAND_HEIGHT"] = str(bh)
        print(f"seed {seed} case {done}: {spec} band height {bh}", flush=True)
        try:
            layer = check_layer(W.make_conv_inputs(spec, 1500 + 100 * seed + done),
                                out_mode=rnd.choice([B.SC_OUT_ZERO_FILL, B.SC_OUT_ZERO_FILL, B.SC_OUT_SCATTER_ONLY]))
        finally:
            os.environ.pop("SPARSE_CONV_BAND_HEIGHT", None)
        assert B.sparse_conv_plan_kernel(layer.plan, 0) == "band_row_segments"
        done += 1


def test_refreshed_mask_and_filters_on_one_plan():
    """Alg. 1, main loop, on a stem-like layer: new row masks and new filters go into the same plan step by step
    (sparse_conv_plan_set_mask rebuilds the band tables, _set_filters the row-segment packing)."""
    spec = spec_of(2, 3, 38, 48, 64, k=7, s=2, p=3, dtype="bf16", sp=0.5)
    ci = W.make_conv_inputs(spec, 1495)
    layer = R.ConvLayer(spec, ci.w, ci.bias, ci.mask)
    assert B.sparse_conv_plan_kernel(layer.plan, 0) == "band_row_segments"
    x = R.to_device(ci.x, spec.dtype)
    rng = np.random.default_rng(1496)
    keep = int(ci.mask.sum())
    for step in range(3):
        mask = np.zeros(spec.m, np.uint8)
        mask[rng.permutation(spec.m)[:keep]] = 1
        w_step = W.quantize(ci.w + np.float32(0.02) * rng.standard_normal(ci.w.shape).astype(np.float32), spec.dtype)
        B.sparse_conv_plan_set_mask(layer.plan, torch.from_numpy(mask).to("cuda:0"))
        B.sparse_conv_plan_set_filters(layer.plan, R.to_device(w_step, spec.dtype))
        assert np.array_equal(B.plan_row_idx(layer.plan).cpu().numpy(), oracle.compact_rows(mask))
        y = layer.new_output(fill_nan=True)
        layer.sparse(x, y)
        torch.cuda.synchronize()
        ref, absum = oracle.masked_conv2d(spec, ci.x, w_step, ci.bias, mask, want_absum=True)
        g, bits = rows_view(spec, R.to_host_f32(y)), rows_view(spec, R.bits_of(y))
        assert (bits[mask == 0] == 0).all()
        assert_close(g[mask == 1], rows_view(spec, ref)[mask == 1], rows_view(spec, absum)[mask == 1], TOL["bf16"], f"step {step}")
