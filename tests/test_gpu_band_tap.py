"""The tap-pipelined band kernel (3x3 windows, 16-bit types: filters arrive tap by tap under the MFMAs) through the
C ABI against the oracle, alone and fused with a shortcut sum."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import oracle
from paper_2309_06626_amd import binding as B
from paper_2309_06626_amd import runtime as R
from parity import check_layer
from test_gpu_parity import spec_of
from test_gpu_residual import check as check_residual
from test_gpu_residual import spec_of as res_spec_of

pytestmark = pytest.mark.gpu

TAP_CASES = [
    dict(n=2, cin=64, h=20, w=20, cout=64),                          # 8 channel groups per pixel, two filter blocks
    dict(n=3, cin=32, h=17, w=19, cout=32, sp=0.3),                  # 4 groups per pixel, one filter block
    dict(n=2, cin=64, h=18, w=18, cout=128, sp=0.4),                 # two channel tiles per band
    dict(n=2, cin=32, h=21, w=21, cout=48, k=3, s=2, p=1, sp=0.5),   # stride 2, ragged channel tile
    dict(n=1, cin=64, h=15, w=13, cout=64, k=3, p=2, d=2, sp=0.6),   # dilation 2
    dict(n=2, cin=32, h=14, w=14, cout=64, sp=0.0),                  # every row kept
    dict(n=1, cin=64, h=12, w=12, cout=64, sp=0.95),                 # bands with almost no kept rows
    dict(n=2, cin=64, h=9, w=40, cout=32, sp=0.2),                   # one filter block of 64 input channels
    dict(n=1, cin=32, h=30, w=7, cout=64, k=3, p=0, sp=0.5),         # no padding
]


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("mask_mode", ["row", "spatial"])
@pytest.mark.parametrize("case", range(len(TAP_CASES)))
def test_tap_band_kernel(case, mask_mode, dtype, monkeypatch):
    monkeypatch.setenv("SPARSE_CONV_BAND_KERNEL", "tap")
    spec = spec_of(dtype=dtype, mask_mode=mask_mode, **TAP_CASES[case])
    layer = check_layer(W.make_conv_inputs(spec, 1930 + case), tiles=(-1, 0))
    assert B.sparse_conv_plan_kernel(layer.plan, 0) == "band_tap"
    assert B.sparse_conv_plan_kernel(layer.plan, 1) == "band_tap"


@pytest.mark.parametrize("bh,n,h,w,sp", [(1, 3, 20, 24, 0.5), (3, 2, 20, 40, 0.3), (7, 2, 30, 56, 0.5), (7, 2, 30, 56, 0.1),
                                         (9, 1, 30, 56, 0.0), (6, 40, 12, 16, 0.6), (4, 2, 13, 100, 0.5)])
def test_tap_band_kernel_band_heights(bh, n, h, w, sp, monkeypatch):
    """Bands of 24 .. 512 pixels: one or two 32-row blocks per wavefront, wavefronts without a block, a ragged last
    band, more bands than compute units."""
    monkeypatch.setenv("SPARSE_CONV_BAND_KERNEL", "tap")
    monkeypatch.setenv("SPARSE_CONV_BAND_HEIGHT", str(bh))
    spec = spec_of(n, 64, h, w, 64, dtype="bf16", sp=sp)
    layer = check_layer(W.make_conv_inputs(spec, 1960 + bh + h), tiles=(-1, 0),
                        sample_rows=None if n * h * w < 5000 else 500)
    tm, tn, wgs = B.sparse_conv_plan_tiles(layer.plan, 0)
    assert (tm, tn) == (-bh, 64) and wgs == n * ((h + bh - 1) // bh)
    assert B.sparse_conv_plan_kernel(layer.plan, 0) == "band_tap"


def test_tap_band_kernel_scatter_only_one_row_and_no_row(monkeypatch):
    monkeypatch.setenv("SPARSE_CONV_BAND_KERNEL", "tap")
    spec = spec_of(2, 32, 16, 16, 64, dtype="bf16", sp=0.5)
    ci = W.make_conv_inputs(spec, 1941)
    layer = check_layer(ci, tiles=(-1, 0), out_mode=B.SC_OUT_SCATTER_ONLY)
    assert B.sparse_conv_plan_kernel(layer.plan, 0) == "band_tap"
    ci.mask[:] = 0
    ci.mask[100] = 1
    check_layer(ci, tiles=(-1, 0), check_count=False)
    ci.mask[:] = 0
    check_layer(ci, tiles=(-1, 0), check_count=False)


def test_tap_band_kernel_without_bias_and_relu(monkeypatch):
    monkeypatch.setenv("SPARSE_CONV_BAND_KERNEL", "tap")
    for bias, relu in [(False, False), (True, False), (False, True)]:
        spec = spec_of(2, 64, 14, 14, 64, dtype="f16", bias=bias, relu=relu, sp=0.5)
        layer = check_layer(W.make_conv_inputs(spec, 1950), tiles=(-1, 0))
        assert B.sparse_conv_plan_kernel(layer.plan, 0) == "band_tap"


def test_tap_band_kernel_on_the_benchmark_layer_at_full_size(monkeypatch):
    """configs[1] at every sparsity, every row through the oracle, in the launch shape bench.py times."""
    monkeypatch.setenv("SPARSE_CONV_BAND_KERNEL", "tap")
    for sp in (0.0, 0.25, 0.5, 0.7):
        ci = W.make_conv_inputs(W.config2(sp), W.base_seed(2))
        layer = check_layer(ci, tiles=(-1, 0))
        assert B.sparse_conv_plan_kernel(layer.plan, 0) == "band_tap"
        assert B.sparse_conv_plan_tiles(layer.plan, 0) == (-7, 64, 256)


def test_a_non_finite_input_value_reaches_only_the_windows_that_contain_it(monkeypatch):
    """Padded taps and absent rows read a zeroed group of LDS, never a neighbour's pixel times zero."""
    monkeypatch.setenv("SPARSE_CONV_BAND_KERNEL", "tap")
    spec = spec_of(1, 64, 12, 12, 64, dtype="bf16", sp=0.0, relu=False)
    ci = W.make_conv_inputs(spec, 1957)
    x = ci.x.copy()
    x[0, 0, 0, :] = np.inf
    x[0, 7, 11, 5] = -np.inf
    layer = R.ConvLayer(spec, ci.w, ci.bias, ci.mask)
    assert B.sparse_conv_plan_kernel(layer.plan, 0) == "band_tap"
    y = layer.new_output(fill_nan=True)
    layer.sparse(R.to_device(x, "bf16"), y)
    torch.cuda.synchronize()
    got = R.to_host_f32(y)
    with np.errstate(invalid="ignore", over="ignore"):
        ref = oracle.masked_conv2d(spec, x, ci.w, ci.bias, ci.mask)
    assert np.array_equal(np.isfinite(got), np.isfinite(ref))
    assert not np.isfinite(ref).all() and np.isfinite(ref).sum() > ref.size // 2


RES_CASES = [
    dict(n=2, cin=64, h=20, w=20, cout=64),
    dict(n=3, cin=32, h=17, w=19, cout=32, sp=0.3),
    dict(n=2, cin=64, h=18, w=18, cout=128, sp=0.4),
    dict(n=2, cin=32, h=21, w=21, cout=48, k=3, s=2, p=1, sp=0.5),
    dict(n=2, cin=32, h=14, w=14, cout=64, sp=0.0),
    dict(n=1, cin=64, h=12, w=12, cout=64, sp=0.95),
    dict(n=2, cin=64, h=16, w=16, cout=64, relu=True),
]


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("mask_mode", ["row", "spatial"])
@pytest.mark.parametrize("post_relu", [False, True])
@pytest.mark.parametrize("case", range(len(RES_CASES)))
def test_fused_shortcut_in_the_tap_band_kernel(case, post_relu, mask_mode, dtype, monkeypatch):
    monkeypatch.setenv("SPARSE_CONV_BAND_KERNEL", "tap")
    spec = res_spec_of(dtype=dtype, mask_mode=mask_mode, **RES_CASES[case])
    layer = check_residual(spec, 2260 + case, post_relu, want_kernel=("band_tap",))
    assert B.sparse_conv_plan_kernel(layer.plan, 0) == "band_tap" == B.sparse_conv_plan_fused_kernel(layer.plan, 1)


def test_fused_shortcut_in_the_tap_band_kernel_tall_bands_and_scatter_only(monkeypatch):
    monkeypatch.setenv("SPARSE_CONV_BAND_KERNEL", "tap")
    monkeypatch.setenv("SPARSE_CONV_BAND_HEIGHT", "7")
    check_residual(res_spec_of(2, 64, 30, 56, 64, sp=0.2), 2290, True, want_kernel=("band_tap",))
    monkeypatch.delenv("SPARSE_CONV_BAND_HEIGHT")
    check_residual(res_spec_of(2, 64, 20, 20, 64), 2291, False, want_kernel=("band_tap",), out_mode=B.SC_OUT_SCATTER_ONLY)
