"""The masked convolution fused with the shortcut sum that follows it (sparse_conv_run_residual,
dense_conv_run_residual) against the oracle: kept rows within the layer tolerance, dropped rows exactly
post(shortcut)."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import oracle
from paper_2309_06626_amd import binding as B
from paper_2309_06626_amd import runtime as R
from parity import TOL, assert_close, row_mask, rows_view

pytestmark = pytest.mark.gpu


def spec_of(n, cin, h, w, cout, k=3, s=1, p=None, dtype="bf16", layout="nhwc", relu=False, sp=0.5, mask_mode="row"):
    p = k // 2 if p is None else p
    return W.ConvSpec("res", n=n, c_in=cin, h=h, w=w, c_out=cout, kh=k, kw=k, stride_h=s, stride_w=s, pad_h=p, pad_w=p,
                      dtype=dtype, layout=layout, relu=relu, sparsity=sp, mask_mode=mask_mode)


def check(spec, seed, post_relu, want_kernel=None, out_mode=B.SC_OUT_ZERO_FILL, split_k=None, y_compact=False,
          x_compact=False, stream_k=None):
    ci = W.make_conv_inputs(spec, seed)
    layer = R.ConvLayer(spec, ci.w, ci.bias, ci.mask, out_mode=out_mode)
    if split_k:
        B.sparse_conv_plan_set_option(layer.plan, B.SC_OPT_SPLIT_K, split_k)
    if stream_k:
        B.sparse_conv_plan_set_tiles(layer.plan, 0, 64, 128)
        B.sparse_conv_plan_set_tiles(layer.plan, 1, 64, 128)
        B.sparse_conv_plan_set_option(layer.plan, B.SC_OPT_STREAM_K, stream_k)
    rm = row_mask(spec, ci.mask)
    kept = rm == 1
    tol = TOL[spec.dtype]
    dt = B.TORCH_DTYPE[spec.dtype]
    rng = np.random.default_rng(seed + 3)
    res_dense = W.quantize(rng.standard_normal(spec.y_shape()).astype(np.float32), spec.dtype)
    res_rows = rows_view(spec, res_dense)
    x_host = ci.x
    x_dev = R.to_device(ci.x, spec.dtype)
    if x_compact:
        x_dev = R.to_device(np.ascontiguousarray(ci.x.reshape(spec.m, spec.c_in)[kept]), spec.dtype)
        x_host = np.ascontiguousarray(ci.x.reshape(spec.m, spec.c_in)[kept])
    # reference: conv without the layer's rounding, plus shortcut, post activation (dense map)
    conv, absum = oracle.masked_conv2d(spec, ci.x * (rm.reshape(spec.n, spec.ho, spec.wo, 1) if x_compact else 1.0), ci.w,
                                       ci.bias, ci.mask, want_absum=True)
    ref = oracle.masked_conv2d_residual(spec, x_host, ci.w, ci.bias, ci.mask, res_rows[kept] if y_compact else res_dense,
                                        post_relu, x_compact=x_compact, y_compact=y_compact)
    bound = rows_view(spec, absum) + np.abs(res_rows)
    if y_compact:
        res_dev = R.to_device(np.ascontiguousarray(res_rows[kept]), spec.dtype)
        y = torch.full((int(kept.sum()) + 1, spec.c_out), float("nan"), dtype=dt, device="cuda:0")
        B.sparse_conv_run_residual(layer.plan, x_dev, layer.bias, res_dev, y[:-1], post_relu,
                                   B.SC_ROWS_COMPACT if x_compact else B.SC_ROWS_DENSE, B.SC_ROWS_COMPACT)
        torch.cuda.synchronize()
        assert np.isnan(R.to_host_f32(y[-1:])).all()
        assert_close(R.to_host_f32(y[:-1]), ref, bound[kept], tol, "compact, fused shortcut")
        return layer
    res_dev = R.to_device(res_dense, spec.dtype)
    sentinel = float("nan") if out_mode == B.SC_OUT_ZERO_FILL else 7.0
    y = layer.new_output().fill_(sentinel)
    B.sparse_conv_run_residual(layer.plan, x_dev, layer.bias, res_dev, y, post_relu)
    torch.cuda.synchronize()
    if want_kernel:
        assert B.sparse_conv_plan_fused_kernel(layer.plan, 0) in want_kernel
    g, bits = rows_view(spec, R.to_host_f32(y)), rows_view(spec, R.bits_of(y))
    refr = rows_view(spec, ref)
    assert_close(g[kept], refr[kept], bound[kept], tol, "kept rows, fused shortcut")
    if out_mode == B.SC_OUT_ZERO_FILL:
        want = oracle.round_storage(refr, spec.dtype)
        assert np.array_equal(g[~kept], want[~kept]), "dropped rows hold post(shortcut) exactly"
    else:
        assert (g[~kept] == 7.0).all()
    # the shortcut tensor itself is untouched
    assert np.array_equal(R.to_host_f32(res_dev), res_dense)
    # dense run: every row is conv + shortcut
    yd = layer.new_output(fill_nan=True)
    B.sparse_conv_run_residual(layer.plan, R.to_device(ci.x, spec.dtype), layer.bias, res_dev, yd, post_relu, dense=True)
    torch.cuda.synchronize()
    ones = np.ones_like(ci.mask)
    refd = oracle.masked_conv2d_residual(spec, ci.x, ci.w, ci.bias, ones, res_dense, post_relu)
    _, absd = oracle.masked_conv2d(spec, ci.x, ci.w, ci.bias, ones, want_absum=True)
    assert_close(rows_view(spec, R.to_host_f32(yd)), rows_view(spec, refd), rows_view(spec, absd) + np.abs(res_rows), tol,
                 "dense run, fused shortcut")
    return layer


@pytest.mark.parametrize("post_relu", [False, True])
@pytest.mark.parametrize("case", [
    dict(n=2, cin=32, h=14, w=14, cout=64),                              # direct-to-LDS gather
    dict(n=2, cin=64, h=12, w=12, cout=128, sp=0.4),                     # buffer-load gather, two channel tiles
    dict(n=1, cin=128, h=9, w=11, cout=256, k=1, sp=0.6),                # pointwise
    dict(n=2, cin=48, h=10, w=10, cout=24, sp=0.3),                      # 16-byte groups, no multiple of 16 channels
    dict(n=1, cin=64, h=16, w=16, cout=64, s=2),                         # stride 2
    dict(n=3, cin=64, h=20, w=20, cout=64, mask_mode="spatial"),         # a band-kernel layer: fused runs take the tiled kernel
    dict(n=2, cin=19, h=8, w=9, cout=21),                                # element gather and element stores
    dict(n=1, cin=16, h=8, w=8, cout=32, relu=True),                     # the layer's own ReLU acts before the sum
])
@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
def test_fused_shortcut(case, post_relu, dtype):
    check(spec_of(dtype=dtype, **case), 1100 + len(str(case)), post_relu)


def test_fused_shortcut_nchw_fp32():
    check(spec_of(2, 6, 9, 7, 10, dtype="f32", layout="nchw"), 1201, True)


def test_every_row_kept():
    check(spec_of(2, 32, 10, 10, 64, sp=0.0), 1210, True)


@pytest.mark.parametrize("post_relu", [False, True])
def test_no_row_kept_leaves_the_shortcut(post_relu):
    spec = spec_of(2, 32, 10, 10, 64)
    ci = W.make_conv_inputs(spec, 1211)
    layer = R.ConvLayer(spec, ci.w, ci.bias, np.zeros_like(ci.mask), check_count=False)
    assert layer.info["kept"] == 0
    res = W.quantize(np.random.default_rng(5).standard_normal(spec.y_shape()).astype(np.float32), spec.dtype)
    y = layer.new_output(fill_nan=True)
    B.sparse_conv_run_residual(layer.plan, R.to_device(ci.x, spec.dtype), layer.bias, R.to_device(res, spec.dtype), y, post_relu)
    torch.cuda.synchronize()
    assert np.array_equal(R.to_host_f32(y), np.maximum(res, 0.0) if post_relu else res + 0.0)


def test_scatter_only_mode_leaves_dropped_rows_alone():
    check(spec_of(2, 64, 12, 12, 64), 1220, True, out_mode=B.SC_OUT_SCATTER_ONLY)


def test_split_k_with_a_fused_shortcut():
    check(spec_of(2, 128, 14, 14, 128), 1230, True, split_k=3)


@pytest.mark.parametrize("x_compact", [False, True])
@pytest.mark.parametrize("post_relu", [False, True])
def test_compact_rows_with_a_fused_shortcut(x_compact, post_relu):
    """The projection of an inverted-residual block: 1x1, linear, compact in and out, shortcut compact as well."""
    check(spec_of(2, 96, 14, 14, 32, k=1, mask_mode="spatial"), 1240, post_relu, y_compact=True, x_compact=x_compact)
    check(spec_of(1, 144, 9, 9, 24, k=1), 1241, post_relu, y_compact=True, x_compact=x_compact)


BAND_CASES = [
    dict(n=2, cin=64, h=20, w=20, cout=64),                          # 8 channel groups per pixel, two filter blocks
    dict(n=3, cin=32, h=17, w=19, cout=32, sp=0.3),                  # 4 groups per pixel, one filter block
    dict(n=2, cin=64, h=18, w=18, cout=128, sp=0.4),                 # two channel tiles per band
    dict(n=2, cin=32, h=21, w=21, cout=48, k=3, s=2, p=1, sp=0.5),   # stride 2, ragged channel tile
    dict(n=2, cin=32, h=14, w=14, cout=64, sp=0.0),                  # every row kept
    dict(n=1, cin=64, h=12, w=12, cout=64, sp=0.95),                 # bands with almost no kept rows
    dict(n=2, cin=64, h=16, w=16, cout=64, relu=True),               # the layer's own ReLU acts before the sum
]


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("mask_mode", ["row", "spatial"])
@pytest.mark.parametrize("post_relu", [False, True])
@pytest.mark.parametrize("case", range(len(BAND_CASES)))
def test_fused_shortcut_in_the_alternating_band_kernel(case, post_relu, mask_mode, dtype, monkeypatch):
    monkeypatch.setenv("SPARSE_CONV_BAND_KERNEL", "alternating")
    spec = spec_of(dtype=dtype, mask_mode=mask_mode, **BAND_CASES[case])
    layer = check(spec, 1260 + case, post_relu, want_kernel=("band_alternating",))
    assert B.sparse_conv_plan_kernel(layer.plan, 0) == "band_alternating" == B.sparse_conv_plan_fused_kernel(layer.plan, 1)


@pytest.mark.parametrize("bh,n,h,w,sp", [(7, 3, 23, 20, 0.5), (5, 2, 17, 9, 0.4), (7, 40, 56, 16, 0.5), (1, 8, 100, 8, 0.5)])
def test_fused_shortcut_in_the_alternating_band_kernel_split_bands_and_many_steps(bh, n, h, w, sp, monkeypatch):
    monkeypatch.setenv("SPARSE_CONV_BAND_KERNEL", "alternating")
    monkeypatch.setenv("SPARSE_CONV_BAND_HEIGHT", f"{bh},split" if bh > 1 else str(bh))
    spec = spec_of(n, 64 if bh > 1 else 32, h, w, 64, dtype="bf16", sp=sp)
    check(spec, 1280 + bh + h, True, want_kernel=("band_alternating",))


def test_fused_shortcut_in_the_alternating_band_kernel_scatter_only(monkeypatch):
    monkeypatch.setenv("SPARSE_CONV_BAND_KERNEL", "alternating")
    check(spec_of(2, 64, 20, 20, 64), 1290, False, want_kernel=("band_alternating",), out_mode=B.SC_OUT_SCATTER_ONLY)


def test_other_band_kernels_hand_a_fused_launch_to_the_tiled_kernel():
    spec = spec_of(2, 16, 20, 20, 64)             # two channel groups per pixel: the plain one-band-per-workgroup kernel
    layer = check(spec, 1291, True, want_kernel=("tile_lds_direct", "tile_masked_store"))
    assert B.sparse_conv_plan_kernel(layer.plan, 0) == "band"


def test_refusals():
    spec = W.ConvSpec("dw", n=1, c_in=16, h=8, w=8, c_out=16, dtype="bf16", sparsity=0.5, groups=16)
    ci = W.make_conv_inputs(spec, 1250)
    layer = R.ConvLayer(spec, ci.w, ci.bias, ci.mask)
    x = R.to_device(ci.x, "bf16")
    y, r = layer.new_output(), layer.new_output()
    with pytest.raises(B.ScError):
        B.sparse_conv_run_residual(layer.plan, x, layer.bias, r, y)          # depthwise plans have no fused form
    spec = spec_of(1, 16, 8, 8, 16)
    ci = W.make_conv_inputs(spec, 1251)
    layer = R.ConvLayer(spec, ci.w, ci.bias, ci.mask)
    x, y = R.to_device(ci.x, "bf16"), layer.new_output()
    with pytest.raises(ValueError):
        B.sparse_conv_run_residual(layer.plan, x, layer.bias, y, y)          # the shortcut must not overlap y
    assert B.lib().sparse_conv_run_residual(layer.plan.handle, x.data_ptr(), 0, layer.bias.data_ptr(), None, 0, y.data_ptr(), 0,
                                           None) == B.SC_ERR_NULL


@pytest.mark.parametrize("dense", [False, True])
def test_resnet18_stack_with_shortcut_sums_fused_into_their_convolutions(dense):
    """The ResNet18 op list with every sum the planner accepts riding in its convolution's epilogue: the sums'
    results against the oracle's interpreter (which rounds the convolution and the sum separately, so the fused
    run differs by at most that one intermediate rounding -- well inside the layer tolerance), the unfused
    tensors bit for bit against the unfused runner, and once more as a graph replay."""
    ops = W.config3(batch=2)
    bs = W.base_seed(3)
    params = {}

    def layer_inputs(spec):
        if spec.name not in params:
            ci = W.make_conv_inputs(spec, bs, x=np.zeros(1, np.float32))
            w, bias, mask = ci.w, ci.bias, ci.mask
            params[spec.name] = (w, bias, np.ones_like(mask) if dense else mask)
        return params[spec.name]

    host = {"input": W.gen_activations(W.network_input_shape(ops), bs, "bf16")}
    layers = {}
    for s in W.conv_specs(ops):
        w, bias, _ = layer_inputs(s)
        layers[s.name] = R.ConvLayer(s, w, bias, W.make_conv_inputs(s, bs, x=np.zeros(1, np.float32)).mask)
    x = R.to_device(host["input"], "bf16")
    net = R.NetworkRunner(ops, {"input": x}, layers, dense=dense, fuse_shortcuts=True)
    sums = [op.out for op in ops if op.kind in ("add", "add_relu")]
    assert net.fusions and set(net.fusions) <= set(sums)
    fused_convs = {v[0] for v in net.fusions.values()}
    for op in ops:
        if op.kind == "conv" and op.spec.name in fused_convs:
            assert op.out not in net.tensors                 # never materialised
    ref = oracle.run_network(ops, host, layer_inputs)
    tol = TOL["bf16"]

    def check():
        torch.cuda.synchronize()
        for op in ops:
            if op.out not in net.tensors:
                continue
            g, r = R.to_host_f32(net.tensors[op.out]), ref[op.out]
            nr = np.linalg.norm(r.astype(np.float64))
            err = np.linalg.norm(g.astype(np.float64) - r.astype(np.float64)) / max(nr, 1e-30)
            assert err <= tol, f"{op.out}: normwise {err:.3e}"
            assert np.abs(g - r).max() <= tol * max(np.abs(r).max(), 1e-30), op.out
            if op.kind == "conv" and not dense:
                bits = rows_view(op.spec, R.bits_of(net.tensors[op.out]))
                assert (bits[params[op.spec.name][2] == 0] == 0).all(), f"{op.out}: dropped rows must be zero"

    net.run()
    check()
    first = {name: R.bits_of(net.tensors[name]).copy() for name in sums}
    graph = net.capture()
    for _ in range(2):
        for name in sums:
            net.tensors[name].fill_(float("nan"))
        graph.replay()
        check()
        for name in sums:
            assert np.array_equal(R.bits_of(net.tensors[name]), first[name]), name
