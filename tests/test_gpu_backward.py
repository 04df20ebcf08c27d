"""Backward pass of the masked convolution through the C ABI against the oracle: gradients w.r.t. the
filters and the bias (float, contraction over the kept rows) and w.r.t. the input (layer dtype)."""
import ctypes

import numpy as np
import pytest
import torch

import workloads as W
from oracle import oracle
from paper_2309_06626_amd import binding as B
from paper_2309_06626_amd import runtime as R
from parity import TOL, assert_close

pytestmark = pytest.mark.gpu

# dw and db come out in float: the operands are exact 16-bit values, products are exact in float and only
# the order of the float additions differs from the oracle's double sums.  With n terms the error is at
# most n * 2^-24 of the sum of magnitudes; the layers here add up to ~10^4 terms per element.
TOL_F32_SUMS = 1e-4


def spec_of(n, c_in, hw, c_out, k=3, s=1, p=None, d=1, dtype="bf16", sparsity=0.5, relu=True, mask_mode="row", w=None):
    p = (d * (k - 1)) // 2 if p is None else p
    return W.ConvSpec("bw", n=n, c_in=c_in, h=hw, w=hw if w is None else w, c_out=c_out, kh=k, kw=k, stride_h=s,
                      stride_w=s, pad_h=p, pad_w=p, dil_h=d, dil_w=d, dtype=dtype, relu=relu, sparsity=sparsity,
                      mask_mode=mask_mode)


def run_backward(spec, seed, want_dx=True, mask=None):
    ci = W.make_conv_inputs(spec, seed)
    mask = ci.mask if mask is None else mask
    layer = R.ConvLayer(spec, ci.w, ci.bias, mask, check_count=False)
    bwd = B.sparse_conv_backward_plan(layer.plan, layer.w)
    rng = np.random.default_rng(seed + 1)
    y = oracle.round_storage(oracle.masked_conv2d(spec, ci.x, ci.w, ci.bias, mask), spec.dtype)   # both sides gate on these values
    dy = W.quantize(rng.standard_normal(spec.y_shape()).astype(np.float32), spec.dtype)
    td = B.TORCH_DTYPE[spec.dtype]
    x_d, y_d, dy_d = R.to_device(ci.x, spec.dtype), R.to_device(y, spec.dtype), R.to_device(dy, spec.dtype)
    dx_d = torch.full(spec.x_shape(), float("nan"), dtype=td, device="cuda:0") if want_dx else None
    dw_d = torch.full(spec.w_shape(), float("nan"), dtype=torch.float32, device="cuda:0")
    db_d = torch.full((spec.c_out,), float("nan"), dtype=torch.float32, device="cuda:0")
    B.sparse_conv_backward_run(bwd, x_d, y_d, dy_d, dx_d, dw_d, db_d)
    torch.cuda.synchronize()
    dx, dw, db, dxa, dwa = oracle.masked_conv2d_backward(spec, ci.x, ci.w, y, dy, mask, want_abs=True)
    rm = oracle.row_mask(spec, mask)
    gate = (y.reshape(spec.m, spec.c_out) > 0) if spec.relu else np.ones((spec.m, spec.c_out), bool)
    dba = (np.abs(dy.reshape(spec.m, spec.c_out).astype(np.float64)) * gate * (rm[:, None] == 1)).sum(axis=0)
    assert_close(dw_d.cpu().numpy(), dw, dwa + 1e-30, TOL_F32_SUMS, "dw")
    assert_close(db_d.cpu().numpy(), db, dba + 1e-30, TOL_F32_SUMS, "db")
    if want_dx:
        assert_close(R.to_host_f32(dx_d), dx, dxa + 1e-30, TOL[spec.dtype], "dx")
    # the same call again gives the same bits (fixed order of additions)
    dw2 = torch.empty_like(dw_d)
    db2 = torch.empty_like(db_d)
    B.sparse_conv_backward_run(bwd, x_d, y_d, dy_d, None, dw2, db2)
    torch.cuda.synchronize()
    assert torch.equal(dw2, dw_d) and torch.equal(db2, db_d)
    return layer, bwd, ci


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("shape", [
    dict(n=2, c_in=64, hw=14, c_out=64),                        # one 128 x 128 tile partly filled, K = 576
    dict(n=3, c_in=32, hw=12, c_out=160, sparsity=0.3),         # two channel tiles, ragged second
    dict(n=2, c_in=24, hw=9, c_out=40, relu=False),             # ragged everything, K = 216
    dict(n=2, c_in=128, hw=10, c_out=64, k=1),                  # pointwise
    dict(n=1, c_in=16, hw=20, c_out=32, d=2),                   # dilation 2
    dict(n=2, c_in=32, hw=11, c_out=48, w=7, mask_mode="spatial"),
])
def test_gradients_match_the_oracle(dtype, shape):
    run_backward(spec_of(dtype=dtype, **shape), 801)


@pytest.mark.parametrize("sparsity", [0.0, 0.9, 0.999])
def test_extreme_sparsities(sparsity):
    run_backward(spec_of(2, 32, 16, 64, sparsity=sparsity), 811)


def test_many_rows_and_row_splits():
    """Enough kept rows for several splits of the contraction and many stages per split."""
    run_backward(spec_of(8, 64, 56, 64, sparsity=0.5), 821)
    run_backward(spec_of(16, 32, 28, 32, k=1, sparsity=0.25), 823)


@pytest.mark.parametrize("shape", [
    dict(n=4, c_in=64, hw=28, c_out=128),                        # wide tile, K = 576: three 192-entry tiles, two 256-entry ones
    dict(n=2, c_in=256, hw=14, c_out=256, sparsity=0.5),         # two channel tiles, K = 2304
    dict(n=2, c_in=40, hw=13, c_out=72, sparsity=0.4),           # groups that straddle nothing, ragged tiles (K = 360)
    dict(n=6, c_in=64, hw=20, c_out=64, sparsity=0.0),           # every row kept: identity row map, narrow tile
    dict(n=3, c_in=96, hw=12, c_out=576, k=1, sparsity=0.5),     # pointwise expansion: five channel tiles, one K tile
    dict(n=2, c_in=64, hw=24, c_out=64, relu=False),             # no gate
    dict(n=40, c_in=32, hw=16, c_out=48, sparsity=0.2, mask_mode="spatial"),
])
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_filter_gradient_with_and_without_the_g_map(dtype, shape):
    """dw and db with the input gradient asked for (the kernel reads the g map) and without (it gates dy by y on the fly):
    run_backward checks both against the oracle and that they agree bit for bit."""
    run_backward(spec_of(dtype=dtype, **shape), 851)


@pytest.mark.parametrize("shape", [
    dict(n=2, c_in=32, hw=16, c_out=64, s=2),                   # the forward pass leaves the last input row unused
    dict(n=2, c_in=32, hw=15, c_out=64, s=2),                   # every input row used
    dict(n=1, c_in=64, hw=14, c_out=128, k=1, s=2),             # pointwise downsample
    dict(n=1, c_in=16, hw=17, c_out=32, s=3, w=11),             # stride 3, non-square
    dict(n=1, c_in=16, hw=18, c_out=16, k=5, s=2, d=2),         # dilated and strided
])
def test_strided_layers(shape):
    """The input gradient of a strided layer: the g map with zeros interleaved, through the forward kernels."""
    run_backward(spec_of(**shape), 827)


def test_padding_beyond_the_window_reach_has_no_input_gradient_path():
    spec = spec_of(1, 16, 8, 16, k=1, p=1)          # 1x1 window with padding 1: dil*(k-1) - pad < 0
    layer, bwd, ci = run_backward(spec, 829, want_dx=False)
    dx = torch.empty(spec.x_shape(), dtype=torch.bfloat16, device="cuda:0")
    dy = torch.zeros(spec.y_shape(), dtype=torch.bfloat16, device="cuda:0")
    with pytest.raises(B.ScError) as err:
        B.sparse_conv_backward_run(bwd, R.to_device(ci.x, spec.dtype), dy, dy, dx, None, None)
    assert err.value.status == B.SC_ERR_UNSUPPORTED


def test_no_kept_row_gives_zero_gradients():
    spec = spec_of(1, 16, 8, 16)
    ci = W.make_conv_inputs(spec, 829)
    run_backward(spec, 829, mask=np.zeros_like(ci.mask))


def test_backward_follows_a_refreshed_mask_and_refreshed_filters():
    spec = spec_of(2, 32, 14, 64, sparsity=0.5)
    layer, bwd, ci = run_backward(spec, 839)
    mask2 = W.gen_mask(spec.mask_len, W.n_keep(0.5, spec.mask_len), 841)
    w2 = W.quantize(ci.w * np.float32(0.5) + np.float32(0.01), spec.dtype)
    B.sparse_conv_plan_set_mask(layer.plan, torch.from_numpy(mask2).to("cuda:0"))
    w2_d = R.to_device(w2, spec.dtype)
    B.sparse_conv_plan_set_filters(layer.plan, w2_d)
    B.sparse_conv_backward_set_filters(bwd, w2_d)
    rng = np.random.default_rng(843)
    y = oracle.round_storage(oracle.masked_conv2d(spec, ci.x, w2, ci.bias, mask2), spec.dtype)
    dy = W.quantize(rng.standard_normal(spec.y_shape()).astype(np.float32), spec.dtype)
    dx_d = torch.full(spec.x_shape(), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    dw_d = torch.empty(spec.w_shape(), dtype=torch.float32, device="cuda:0")
    db_d = torch.empty((spec.c_out,), dtype=torch.float32, device="cuda:0")
    B.sparse_conv_backward_run(bwd, R.to_device(ci.x, spec.dtype), R.to_device(y, spec.dtype), R.to_device(dy, spec.dtype),
                               dx_d, dw_d, db_d)
    torch.cuda.synchronize()
    dx, dw, db, dxa, dwa = oracle.masked_conv2d_backward(spec, ci.x, w2, y, dy, mask2, want_abs=True)
    assert_close(dw_d.cpu().numpy(), dw, dwa + 1e-30, TOL_F32_SUMS, "dw after refresh")
    assert_close(R.to_host_f32(dx_d), dx, dxa + 1e-30, TOL["bf16"], "dx after refresh")


def test_layers_the_backward_kernels_do_not_cover_are_refused():
    L = B.lib()
    size = ctypes.c_size_t()
    for kw in (dict(c_in=20), dict(c_out=20), dict(layout=B.SC_NCHW), dict(groups=16)):
        args = dict(n=1, c_in=16, h=8, w=8, c_out=16)
        args.update(kw)
        d = B.make_desc(**args)
        assert L.sparse_conv_backward_workspace_bytes(ctypes.byref(d), ctypes.byref(size)) == B.SC_ERR_UNSUPPORTED
    d = B.make_desc(1, 16, 8, 8, 16)
    assert L.sparse_conv_backward_workspace_bytes(ctypes.byref(d), ctypes.byref(size)) == B.SC_OK and size.value > 0
    assert L.sparse_conv_backward_workspace_bytes(ctypes.byref(d), None) == B.SC_ERR_NULL
    assert L.sparse_conv_backward_run(None, None, None, None, None, None, None, None) == B.SC_ERR_NULL


# float layers: operands and products round in float on the device; with n terms per element the error of a sum is
# about sqrt(n) * 2^-24 of its terms' magnitudes (a few thousand terms here), inside the 1e-5 the float forward pass
# is held to
@pytest.mark.parametrize("shape", [
    dict(n=2, c_in=16, hw=16, c_out=16),                         # the float layer of the smallest configuration, batch 2
    dict(n=2, c_in=64, hw=14, c_out=64, sparsity=0.3),           # one tile of each operand, K = 576
    dict(n=3, c_in=24, hw=9, c_out=40, relu=False),              # ragged tiles in both directions
    dict(n=2, c_in=128, hw=10, c_out=72, k=1),                   # pointwise, two channel tiles
    dict(n=2, c_in=32, hw=15, c_out=64, s=2),                    # strided: zero-interleaved g map for dx
    dict(n=1, c_in=16, hw=20, c_out=32, d=2),                    # dilation 2
    dict(n=2, c_in=32, hw=11, c_out=48, w=7, mask_mode="spatial"),
    dict(n=4, c_in=32, hw=28, c_out=32, sparsity=0.5),           # several row splits
    dict(n=2, c_in=16, hw=8, c_out=16, sparsity=1.0),            # nothing kept
])
def test_float_layers(shape, monkeypatch):
    import sys
    monkeypatch.setattr(sys.modules[__name__], "TOL_F32_SUMS", 1e-5)
    run_backward(spec_of(dtype="f32", **shape), 871)


def test_float_training_steps_follow_the_oracles_steps():
    """Alg. 1 main loop on a float layer, three steps on both sides: getMask draws the step's mask from a fresh score,
    maskedForward, a squared-error loss against a fixed target (dy = y - target), backward, a plain gradient step on the
    filters and the bias.  Each side feeds on its own previous weights; after three steps they still agree."""
    from oracle import mask_oracle as MO
    spec = W.ConvSpec("train32", n=2, c_in=16, h=16, w=16, c_out=16, dtype="f32", sparsity=0.5, mask_mode="spatial")
    ci = W.make_conv_inputs(spec, 881)
    rng = np.random.default_rng(883)
    target = rng.standard_normal(spec.y_shape()).astype(np.float32)
    lr = np.float32(1e-3)
    w_ref, b_ref = ci.w.astype(np.float64), ci.bias.astype(np.float64)
    w_dev, b_dev = torch.from_numpy(ci.w).to("cuda:0"), torch.from_numpy(ci.bias).to("cuda:0")
    layer = R.ConvLayer(spec, ci.w, ci.bias, ci.mask)
    bwd = B.sparse_conv_backward_plan(layer.plan, w_dev)
    x_d, t_d = torch.from_numpy(ci.x).to("cuda:0"), torch.from_numpy(target).to("cuda:0")
    dw_d = torch.empty(spec.w_shape(), dtype=torch.float32, device="cuda:0")
    db_d = torch.empty(spec.c_out, dtype=torch.float32, device="cuda:0")
    for step in range(3):
        score = W.gen_score(64, 64, seed=890 + step)
        mask_d = B.sparse_mask_generate(torch.from_numpy(score).to("cuda:0"), spec.ho, spec.wo, spec.sparsity)
        mask = MO.layer_mask(score, spec.ho, spec.wo, np.float32(spec.sparsity)).reshape(-1)
        assert np.array_equal(mask_d.cpu().numpy().reshape(-1), mask)
        # device side
        B.sparse_conv_plan_set_mask(layer.plan, mask_d)
        B.sparse_conv_plan_set_filters(layer.plan, w_dev)
        B.sparse_conv_backward_set_filters(bwd, w_dev)
        y_d = B.sparse_conv_run(layer.plan, x_d, b_dev, layer.new_output())
        dy_d = y_d - t_d
        B.sparse_conv_backward_run(bwd, x_d, y_d, dy_d, None, dw_d, db_d)
        w_dev = w_dev - lr * dw_d
        b_dev = b_dev - lr * db_d
        # oracle side (float weights as a float training loop holds them, sums in double)
        w32, b32 = w_ref.astype(np.float32), b_ref.astype(np.float32)
        y = oracle.round_storage(oracle.masked_conv2d(spec, ci.x, w32, b32, mask), "f32")
        _, dw, db = oracle.masked_conv2d_backward(spec, ci.x, w32, y, (y - target).astype(np.float32), mask)
        w_ref = (w32 - lr * dw.astype(np.float32)).astype(np.float64)
        b_ref = (b32 - lr * db.astype(np.float32)).astype(np.float64)
    torch.cuda.synchronize()
    scale = np.abs(w_ref).max()
    assert np.abs(w_dev.cpu().numpy() - w_ref).max() <= 1e-5 * scale
    assert np.abs(b_dev.cpu().numpy() - b_ref).max() <= 1e-5 * max(np.abs(b_ref).max(), 1.0)
    assert np.abs(w_ref - ci.w).max() > 1e-4 * scale          # the steps really moved the weights
