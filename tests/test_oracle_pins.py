"""Pins for the CPU oracle: it is checked against things other than itself.

* a library routine (torch.nn.functional.conv2d in float64) for the unmasked convolution;
* the paper's own three-stage pipeline written out in numpy (explicit lowering matrix,
  skipped rows, dense matmul on fewer rows, backward in-place expansion; Sec. 3.2, Alg. 2);
* closed forms, linearity, locality of a masked window (Fig. 2), exact zeros at dropped
  positions (Alg. 2), kept-row counts (Sec. 3.2) from tests/golden/kept_counts.txt.
"""
import itertools
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import workloads as W
from oracle import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rand_inputs(spec, seed, positive=False):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal(spec.x_shape()).astype(np.float32)
    w = rng.standard_normal(spec.w_shape()).astype(np.float32)
    if positive:
        x, w = np.abs(x), np.abs(w)
    b = rng.standard_normal(spec.c_out).astype(np.float32) if spec.has_bias else None
    keep = W.n_keep(spec.sparsity, spec.mask_len)
    mask = W.gen_mask(spec.mask_len, keep, seed + 7)
    return x, w, b, mask


def torch_conv(spec, x, w, b):
    """Unmasked convolution by the library routine, float64, returned as [N,Ho,Wo,Cout]."""
    xt = torch.from_numpy(x).double()
    wt = torch.from_numpy(w).double()
    if spec.layout == "nhwc":
        xt = xt.permute(0, 3, 1, 2)
        wt = wt.permute(0, 3, 1, 2)
    bt = torch.from_numpy(b).double() if b is not None else None
    y = F.conv2d(xt, wt, bt, stride=(spec.stride_h, spec.stride_w), padding=(spec.pad_h, spec.pad_w),
                 dilation=(spec.dil_h, spec.dil_w))
    if spec.relu:
        y = torch.relu(y)
    return y.permute(0, 2, 3, 1).contiguous().numpy()


def to_rows(spec, y):
    """[M, Cout] view of an output in the spec's layout."""
    if spec.layout == "nchw":
        y = np.transpose(y, (0, 2, 3, 1))
    return np.ascontiguousarray(y).reshape(spec.m, spec.c_out)


def row_mask(spec, mask):
    return np.tile(mask, spec.n) if spec.mask_mode == "spatial" else mask


GEOMS = [
    # n, cin, h, w, cout, kh, kw, sh, sw, ph, pw, dh, dw
    (1, 3, 5, 5, 2, 3, 3, 1, 1, 1, 1, 1, 1),
    (2, 5, 7, 9, 3, 3, 3, 1, 1, 1, 1, 1, 1),
    (1, 4, 9, 6, 5, 1, 1, 1, 1, 0, 0, 1, 1),
    (3, 2, 8, 11, 4, 2, 3, 2, 1, 0, 1, 1, 1),
    (1, 3, 13, 10, 6, 7, 7, 2, 2, 3, 3, 1, 1),
    (2, 6, 9, 9, 2, 3, 3, 2, 2, 1, 1, 2, 2),
    (1, 2, 12, 7, 3, 3, 2, 1, 2, 3, 0, 2, 1),
    (2, 7, 6, 6, 9, 1, 1, 2, 2, 0, 0, 1, 1),
    (1, 1, 4, 4, 1, 2, 2, 1, 1, 0, 0, 1, 1),
]


def make_spec(g, layout="nhwc", bias=True, relu=False, s=0.4, mask_mode="row"):
    n, cin, h, w, cout, kh, kw, sh, sw, ph, pw, dh, dw = g
    return W.ConvSpec("t", n=n, c_in=cin, h=h, w=w, c_out=cout, kh=kh, kw=kw, stride_h=sh, stride_w=sw,
                      pad_h=ph, pad_w=pw, dil_h=dh, dil_w=dw, dtype="f32", layout=layout, has_bias=bias,
                      relu=relu, sparsity=s, mask_mode=mask_mode)


# ---------------------------------------------------------------------------------------
# 1. library routine: sparsity 0 is the plain convolution; any mask = dense (.) mask
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("g", GEOMS)
@pytest.mark.parametrize("layout", ["nhwc", "nchw"])
@pytest.mark.parametrize("bias,relu", [(False, False), (True, True)])
def test_matches_library_conv2d(g, layout, bias, relu):
    spec = make_spec(g, layout, bias, relu, s=0.0)
    x, w, b, mask = rand_inputs(spec, 11)
    assert mask.all()
    ref = torch_conv(spec, x, w, b).reshape(spec.m, spec.c_out)
    got = to_rows(spec, oracle.masked_conv2d(spec, x, w, b, mask))
    np.testing.assert_allclose(got, ref, rtol=3e-7, atol=1e-7)

    spec_s = spec.with_(sparsity=0.4)
    mask = W.gen_mask(spec_s.mask_len, W.n_keep(0.4, spec_s.mask_len), 5)
    got = to_rows(spec_s, oracle.masked_conv2d(spec_s, x, w, b, mask))
    np.testing.assert_allclose(got, ref * mask[:, None], rtol=3e-7, atol=1e-7)
    assert (got[mask == 0].view(np.uint32) == 0).all()


# ---------------------------------------------------------------------------------------
# 2. the paper's pipeline, brute force: lowering matrix -> skip rows -> matmul -> expansion
# ---------------------------------------------------------------------------------------
def lowered_matrix(spec, x):
    """Explicit lowering (one row per output position, K = kh*kw*Cin entries, tap-major)."""
    xn = x if spec.layout == "nhwc" else np.transpose(x, (0, 2, 3, 1))
    a = np.zeros((spec.m, spec.kh, spec.kw, spec.c_in), dtype=np.float64)
    for n, oy, ox in itertools.product(range(spec.n), range(spec.ho), range(spec.wo)):
        r = (n * spec.ho + oy) * spec.wo + ox
        for ky, kx in itertools.product(range(spec.kh), range(spec.kw)):
            iy = oy * spec.stride_h - spec.pad_h + ky * spec.dil_h
            ix = ox * spec.stride_w - spec.pad_w + kx * spec.dil_w
            if 0 <= iy < spec.h and 0 <= ix < spec.w:
                a[r, ky, kx, :] = xn[n, iy, ix, :]
    return a.reshape(spec.m, spec.k)


def alg2_pipeline(spec, x, w, b, mask):
    a = lowered_matrix(spec, x)
    wm = w if spec.layout == "nhwc" else np.transpose(w, (0, 2, 3, 1))
    bmat = wm.reshape(spec.c_out, spec.k).astype(np.float64).T
    rm = row_mask(spec, mask)
    kept_rows = [r for r in range(spec.m) if rm[r] == 1]          # indirection init, ascending
    out = np.full((spec.m, spec.c_out), np.nan)
    compact = a[kept_rows] @ bmat                                   # dense GEMM on fewer rows
    if b is not None:
        compact = compact + b.astype(np.float64)[None, :]
    if spec.relu:
        compact = np.maximum(compact, 0.0)
    out[: len(kept_rows)] = compact                                 # GEMM output sits at the front
    idx = len(kept_rows) - 1
    for r in range(spec.m - 1, -1, -1):                             # post-process, walking backwards
        if rm[r] == 0:
            out[r] = 0.0
        else:
            out[r] = out[idx]
            idx -= 1
    assert idx == -1
    return out


@pytest.mark.parametrize("g", GEOMS)
@pytest.mark.parametrize("layout", ["nhwc", "nchw"])
@pytest.mark.parametrize("mask_mode", ["row", "spatial"])
def test_matches_paper_pipeline_bruteforce(g, layout, mask_mode):
    spec = make_spec(g, layout, bias=True, relu=True, s=0.35, mask_mode=mask_mode)
    x, w, b, mask = rand_inputs(spec, 23)
    ref = alg2_pipeline(spec, x, w, b, mask)
    got = to_rows(spec, oracle.masked_conv2d(spec, x, w, b, mask))
    np.testing.assert_allclose(got, ref, rtol=3e-7, atol=1e-7)


def paper_stage_two(spec, x, w, b, mask):
    """Stage (ii) of Sec. 3.2 alone: the GEMM over the kept rows of the explicit lowering matrix."""
    a = lowered_matrix(spec, x)
    bmat = w.reshape(spec.c_out, spec.k).astype(np.float64).T
    rm = row_mask(spec, mask)
    compact = a[rm == 1] @ bmat
    if b is not None:
        compact = compact + b.astype(np.float64)[None, :]
    return np.maximum(compact, 0.0) if spec.relu else compact


@pytest.mark.parametrize("g", GEOMS)
@pytest.mark.parametrize("mask_mode", ["row", "spatial"])
def test_compact_output_is_the_gemm_result_before_expansion(g, mask_mode):
    spec = make_spec(g, "nhwc", bias=True, relu=True, s=0.35, mask_mode=mask_mode)
    x, w, b, mask = rand_inputs(spec, 29)
    got = oracle.masked_conv2d_compact(spec, x, w, b, mask, y_compact=True)
    ref = paper_stage_two(spec, x, w, b, mask)
    assert got.shape == ref.shape == (int(row_mask(spec, mask).sum()), spec.c_out)
    np.testing.assert_allclose(got, ref, rtol=3e-7, atol=1e-7)


def test_expansion_of_compact_rows_is_the_backward_walk_of_alg2():
    rng = np.random.default_rng(31)
    rm = W.gen_mask(40, 23, 3)
    compact = rng.standard_normal((23, 5)).astype(np.float32)
    out = np.full((40, 5), np.nan, dtype=np.float32)
    out[:23] = compact
    idx = 22
    for r in range(39, -1, -1):                   # Alg. 2: from the last pixel to the first, in place
        if rm[r] == 0:
            out[r] = 0.0
        else:
            out[r] = out[idx]
            idx -= 1
    got = oracle.from_compact(compact, rm, (40, 5))
    assert np.array_equal(got.view(np.uint32), out.view(np.uint32))
    assert np.array_equal(oracle.to_compact(got, rm), compact)


def test_pointwise_layer_on_compact_input_is_a_plain_matrix_product():
    """A 1x1 stride-1 layer reads only the pixel itself: on the kept rows it is X_kept @ W^T + b."""
    spec = make_spec(GEOMS[2], "nhwc", bias=True, relu=False, s=0.4)
    x, w, b, mask = rand_inputs(spec, 37)
    rm = row_mask(spec, mask)
    x[...] = np.where(rm.reshape(spec.n, spec.h, spec.w, 1) == 1, x, 0.0)      # the producer left zeros there
    xc = oracle.to_compact(x, rm)
    ref = xc.astype(np.float64) @ w.reshape(spec.c_out, spec.c_in).astype(np.float64).T + b.astype(np.float64)
    got = oracle.masked_conv2d_compact(spec, xc, w, b, mask, x_compact=True, y_compact=True)
    np.testing.assert_allclose(got, ref, rtol=3e-7, atol=1e-7)
    dense = oracle.masked_conv2d_compact(spec, xc, w, b, mask, x_compact=True)
    assert np.array_equal(dense, oracle.masked_conv2d(spec, x, w, b, mask))
    # garbage at the dropped pixels of a dense input does not reach the kept rows either
    x2 = np.where(rm.reshape(spec.n, spec.h, spec.w, 1) == 1, x, np.float32(1e6))
    assert np.array_equal(oracle.masked_conv2d(spec, x2, w, b, mask), dense)


def test_spatial_mask_is_row_mask_tiled():
    spec = make_spec(GEOMS[3], s=0.5, mask_mode="spatial")
    x, w, b, mask = rand_inputs(spec, 3)
    y_sp = oracle.masked_conv2d(spec, x, w, b, mask)
    y_row = oracle.masked_conv2d(spec.with_(mask_mode="row"), x, w, b, np.tile(mask, spec.n))
    assert np.array_equal(y_sp.view(np.uint32), y_row.view(np.uint32))


# ---------------------------------------------------------------------------------------
# 3. closed forms
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("g", [GEOMS[1], GEOMS[4], GEOMS[5], GEOMS[6]])
def test_all_ones_counts_inbounds_taps(g):
    spec = make_spec(g, bias=False, relu=False, s=0.3)
    x = np.ones(spec.x_shape(), np.float32)
    w = np.ones(spec.w_shape(), np.float32)
    mask = W.gen_mask(spec.m, W.n_keep(0.3, spec.m), 1)
    y = to_rows(spec, oracle.masked_conv2d(spec, x, w, None, mask))
    for r in range(spec.m):
        oy, ox = (r // spec.wo) % spec.ho, r % spec.wo
        ny = sum(0 <= oy * spec.stride_h - spec.pad_h + ky * spec.dil_h < spec.h for ky in range(spec.kh))
        nx = sum(0 <= ox * spec.stride_w - spec.pad_w + kx * spec.dil_w < spec.w for kx in range(spec.kw))
        want = float(spec.c_in * ny * nx) if mask[r] else 0.0
        assert (y[r] == want).all()


@pytest.mark.parametrize("layout", ["nhwc", "nchw"])
def test_centre_tap_identity_returns_masked_input(layout):
    c = 5
    spec = W.ConvSpec("id", n=2, c_in=c, h=6, w=7, c_out=c, dtype="f32", layout=layout, has_bias=False,
                      relu=False, sparsity=0.5)
    x = np.random.default_rng(0).standard_normal(spec.x_shape()).astype(np.float32)
    w = np.zeros(spec.w_shape(), np.float32)
    for i in range(c):
        if layout == "nhwc":
            w[i, 1, 1, i] = 1.0
        else:
            w[i, i, 1, 1] = 1.0
    mask = W.gen_mask(spec.m, spec.m // 2, 2)
    y = to_rows(spec, oracle.masked_conv2d(spec, x, w, None, mask))
    assert np.array_equal(y, to_rows(spec, x) * mask[:, None])


def test_off_centre_tap_shifts_the_right_way():
    # single tap at (ky, kx) = (0, 2) of a 3x3 window with pad 1: y[oy, ox] = x[oy-1, ox+1]
    spec = W.ConvSpec("sh", n=1, c_in=1, h=5, w=6, c_out=1, dtype="f32", has_bias=False, relu=False, sparsity=0.0)
    x = np.arange(30, dtype=np.float32).reshape(1, 5, 6, 1) + 1
    w = np.zeros((1, 3, 3, 1), np.float32)
    w[0, 0, 2, 0] = 1.0
    y = oracle.masked_conv2d(spec, x, w, None, np.ones(30, np.uint8))[0, :, :, 0]
    want = np.zeros((5, 6), np.float32)
    want[1:, :5] = x[0, :4, 1:, 0]
    assert np.array_equal(y, want)


def test_pointwise_identity_copies_kept_rows():
    c = 4
    spec = W.ConvSpec("pw", n=2, c_in=c, h=5, w=3, c_out=c, kh=1, kw=1, pad_h=0, pad_w=0, dtype="f32",
                      has_bias=False, relu=False, sparsity=0.4)
    x = np.random.default_rng(4).standard_normal(spec.x_shape()).astype(np.float32)
    w = np.eye(c, dtype=np.float32).reshape(c, 1, 1, c)
    mask = W.gen_mask(spec.m, W.n_keep(0.4, spec.m), 9)
    y = oracle.masked_conv2d(spec, x, w, None, mask).reshape(spec.m, c)
    assert np.array_equal(y, x.reshape(spec.m, c) * mask[:, None])


def test_weight_operand_not_transposed():
    # Cin != Cout, 1x1: y[r, co] = sum_ci x[r, ci] * w[co, ci]
    spec = W.ConvSpec("tr", n=1, c_in=3, h=2, w=2, c_out=2, kh=1, kw=1, pad_h=0, pad_w=0, dtype="f32",
                      has_bias=False, relu=False, sparsity=0.0)
    x = np.array([[1, 2, 3], [4, 5, 6], [7, 8, 9], [1, 0, -1]], np.float32).reshape(1, 2, 2, 3)
    w = np.array([[1, 0, 2], [0, -1, 1]], np.float32).reshape(2, 1, 1, 3)
    y = oracle.masked_conv2d(spec, x, w, None, np.ones(4, np.uint8)).reshape(4, 2)
    assert np.array_equal(y, np.array([[7, 1], [16, 1], [25, 1], [-1, -1]], np.float32))


# ---------------------------------------------------------------------------------------
# 4. linearity, bias, ReLU
# ---------------------------------------------------------------------------------------
def test_linearity_and_bias():
    spec = make_spec(GEOMS[1], bias=False, relu=False, s=0.4)
    x1, w, _, mask = rand_inputs(spec, 31)
    x2 = np.random.default_rng(32).standard_normal(spec.x_shape()).astype(np.float32)
    a = np.float32(0.5)  # exact scaling
    y1 = oracle.masked_conv2d(spec, x1, w, None, mask).astype(np.float64)
    y2 = oracle.masked_conv2d(spec, x2, w, None, mask).astype(np.float64)
    y12 = oracle.masked_conv2d(spec, a * x1 + x2, w, None, mask).astype(np.float64)
    np.testing.assert_allclose(y12, 0.5 * y1 + y2, rtol=1e-5, atol=2e-6)

    spec_b = spec.with_(has_bias=True)
    b = np.random.default_rng(33).standard_normal(spec.c_out).astype(np.float32)
    yb = to_rows(spec_b, oracle.masked_conv2d(spec_b, x1, w, b, mask)).astype(np.float64)
    y0 = to_rows(spec, y1)
    kept = mask == 1
    np.testing.assert_allclose(yb[kept] - y0[kept], np.broadcast_to(b, yb[kept].shape), rtol=0, atol=2e-6)
    assert (yb[~kept] == 0).all()

    spec_r = spec_b.with_(relu=True)
    yr = to_rows(spec_r, oracle.masked_conv2d(spec_r, x1, w, b, mask))
    assert np.array_equal(yr, np.maximum(yb.astype(np.float32), 0))


# ---------------------------------------------------------------------------------------
# 5. Fig. 2: a masked window is local to its own row
# ---------------------------------------------------------------------------------------
def test_masking_a_window_leaves_neighbours_untouched():
    spec = make_spec(GEOMS[1], s=0.0)
    x, w, b, ones = rand_inputs(spec, 41)
    dense = to_rows(spec, oracle.masked_conv2d(spec, x, w, b, ones))
    for r in (0, 7, spec.m // 2, spec.m - 1):
        m = ones.copy()
        m[r] = 0
        y = to_rows(spec, oracle.masked_conv2d(spec, x, w, b, m))
        assert (y[r].view(np.uint32) == 0).all()
        keep = np.arange(spec.m) != r
        assert np.array_equal(y[keep].view(np.uint32), dense[keep].view(np.uint32))


def test_mask_is_row_major_on_a_non_square_map():
    # Ho = 3, Wo = 5; drop position (oy, ox) = (1, 3) -> row 1*5 + 3
    spec = W.ConvSpec("ns", n=1, c_in=2, h=3, w=5, c_out=2, dtype="f32", has_bias=True, relu=False, sparsity=0.0)
    x, w, b, _ = rand_inputs(spec, 5, positive=True)
    b = np.abs(b) + 1
    mask = np.ones(15, np.uint8)
    mask[1 * 5 + 3] = 0
    y = oracle.masked_conv2d(spec, x, w, b, mask)
    zero = (y == 0).all(axis=-1)[0]
    want = np.zeros((3, 5), bool)
    want[1, 3] = True
    assert np.array_equal(zero, want)


def test_dropped_rows_are_plus_zero_even_with_bias():
    spec = make_spec(GEOMS[4], bias=True, relu=False, s=0.6)
    x, w, b, mask = rand_inputs(spec, 17)
    y = to_rows(spec, oracle.masked_conv2d(spec, x, w, b, mask))
    assert (y[mask == 0].view(np.uint32) == 0).all()          # +0.0 bit pattern, no bias
    assert (np.abs(y[mask == 1]).sum(axis=1) > 0).all()


# ---------------------------------------------------------------------------------------
# 6. kept-row count and compaction (Sec. 3.2, Alg. 2 indirection init)
# ---------------------------------------------------------------------------------------
def golden_counts():
    rows = []
    with open(os.path.join(GOLDEN, "kept_counts.txt")) as f:
        for line in f:
            line = line.split("#")[0].split()
            if line:
                rows.append((int(line[0]), float(line[1]), int(line[2]), line[3]))
    return rows


@pytest.mark.parametrize("m,s,kept,kind", golden_counts())
def test_kept_count_golden(m, s, kept, kind):
    assert oracle.kept_count(s, m) == kept
    if kind == "exact":
        assert abs((m - s * m) - kept) < 1e-6


def test_compaction_is_ascending_list_of_ones():
    rng = np.random.default_rng(0)
    for m in (1, 2, 63, 64, 65, 1000, 4097):
        mask = (rng.random(m) < 0.6).astype(np.uint8)
        idx = oracle.compact_rows(mask)
        assert idx.dtype == np.int32
        assert np.array_equal(idx, np.flatnonzero(mask))
        assert (np.diff(idx) > 0).all()
    assert oracle.compact_rows(np.zeros(10, np.uint8)).size == 0
    assert np.array_equal(oracle.compact_rows(np.ones(10, np.uint8)), np.arange(10))
    with pytest.raises(ValueError):
        oracle.compact_rows(np.array([0, 1, 2], np.uint8))


def test_bad_mask_byte_rejected():
    spec = make_spec(GEOMS[0])
    x, w, b, mask = rand_inputs(spec, 1)
    mask = mask.copy()
    mask[3] = 2
    with pytest.raises(ValueError):
        oracle.masked_conv2d(spec, x, w, b, mask)


# ---------------------------------------------------------------------------------------
# 7. helpers: sampled rows, error scale, storage rounding, network glue
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("layout", ["nhwc", "nchw"])
def test_sampled_rows_equal_full(layout):
    spec = make_spec(GEOMS[5], layout, bias=True, relu=True, s=0.3)
    x, w, b, mask = rand_inputs(spec, 51)
    full, absum = oracle.masked_conv2d(spec, x, w, b, mask, want_absum=True)
    rows = np.array([0, 3, spec.m - 1, 5, 5], dtype=np.int64)
    yr, ar = oracle.masked_conv2d_rows(spec, x, w, b, mask, rows, want_absum=True)
    assert np.array_equal(yr, to_rows(spec, full)[rows])
    assert np.array_equal(ar, to_rows(spec, absum)[rows])


def test_absum_is_the_l1_scale():
    spec = make_spec(GEOMS[1], bias=True, relu=False, s=0.3)
    x, w, b, mask = rand_inputs(spec, 61, positive=True)
    b = np.abs(b)
    y, absum = oracle.masked_conv2d(spec, x, w, b, mask, want_absum=True)
    np.testing.assert_allclose(absum, y.astype(np.float64), rtol=1e-6)   # all terms positive
    x2 = -x
    y2, absum2 = oracle.masked_conv2d(spec, x2, w, b, mask, want_absum=True)
    np.testing.assert_allclose(absum2, absum, rtol=1e-12)


def test_storage_rounding_matches_library_casts():
    rng = np.random.default_rng(5)
    a = (rng.standard_normal(50000) * 10.0 ** rng.integers(-8, 5, 50000)).astype(np.float32)
    a[:4] = [0.0, -0.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8]              # ties: to even
    got = oracle.round_storage(a, "bf16")
    ref = torch.from_numpy(a).to(torch.bfloat16).float().numpy()
    assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))
    got = oracle.round_storage(a, "f16")
    with np.errstate(over="ignore"):
        ref = a.astype(np.float16).astype(np.float32)
    assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))
    assert np.array_equal(oracle.round_storage(a, "f32"), a)


def test_network_glue_ops_match_library():
    rng = np.random.default_rng(6)
    x = rng.standard_normal((2, 9, 11, 5)).astype(np.float32)
    ref = F.max_pool2d(torch.from_numpy(x).permute(0, 3, 1, 2), 3, 2, 1).permute(0, 2, 3, 1).numpy()
    assert np.array_equal(oracle.maxpool2d_nhwc(x, 3, 2, 1), ref)
    a, b = x, rng.standard_normal(x.shape).astype(np.float32)
    assert np.array_equal(oracle.add_relu(a, b), np.maximum(a + b, 0))


def test_small_resnet_chain_matches_library_pipeline():
    """The network interpreter wires tensors as the op list says (tiny ResNet18 stack, fp32)."""
    ops = W.config3(batch=1, res=32, sparsity=0.0, dtype="f32")
    bs = 99
    x = W.gen_activations(W.network_input_shape(ops), bs, "f32")
    params = {}

    def layer_inputs(spec):
        if spec.name not in params:
            ci = W.make_conv_inputs(spec, bs, x=np.zeros(1, np.float32))
            params[spec.name] = (ci.w, ci.bias, ci.mask)
        return params[spec.name]

    t = oracle.run_network(ops, {"input": x}, layer_inputs)
    # the same graph through torch, float64
    tt = {"input": torch.from_numpy(x).double().permute(0, 3, 1, 2)}
    for op in ops:
        if op.kind == "conv":
            s = op.spec
            w, b, _ = layer_inputs(s)
            y = F.conv2d(tt[op.src], torch.from_numpy(w).double().permute(0, 3, 1, 2), torch.from_numpy(b).double(),
                         stride=s.stride_h, padding=s.pad_h)
            tt[op.out] = torch.relu(y) if s.relu else y
        elif op.kind == "maxpool":
            tt[op.out] = F.max_pool2d(tt[op.src], 3, 2, 1)
        else:
            tt[op.out] = torch.relu(tt[op.src] + tt[op.src2])
    last = ops[-1].out
    ref = tt[last].permute(0, 2, 3, 1).numpy()
    np.testing.assert_allclose(t[last], ref, rtol=2e-4, atol=2e-5)
    assert t[last].shape == (1, 1, 1, 512)


@pytest.mark.parametrize("post_relu", [False, True])
@pytest.mark.parametrize("y_compact", [False, True])
def test_convolution_with_shortcut_sum_matches_the_library_pipeline(post_relu, y_compact):
    """conv2d by the library, masked, plus the shortcut, ReLU last: the dropped rows of the result hold
    post(shortcut), not zero; a compact result holds the kept rows of that map."""
    spec = W.ConvSpec("r", n=2, c_in=5, h=7, w=6, c_out=4, kh=3, kw=3, pad_h=1, pad_w=1, dtype="f32", relu=False,
                      sparsity=0.4)
    x, w, b, mask = rand_inputs(spec, 71)
    rng = np.random.default_rng(72)
    rm = oracle.row_mask(spec, mask)
    res_dense = rng.standard_normal(spec.y_shape()).astype(np.float32)
    conv = torch_conv(spec, x, w, b).reshape(spec.m, spec.c_out) * rm[:, None]
    want = conv + res_dense.reshape(spec.m, spec.c_out)
    if post_relu:
        want = np.maximum(want, 0.0)
    if y_compact:
        res = np.ascontiguousarray(res_dense.reshape(spec.m, spec.c_out)[rm == 1])
        got = oracle.masked_conv2d_residual(spec, x, w, b, mask, res, post_relu, y_compact=True)
        np.testing.assert_allclose(got, want[rm == 1], rtol=1e-5, atol=1e-6)
    else:
        got = oracle.masked_conv2d_residual(spec, x, w, b, mask, res_dense, post_relu)
        np.testing.assert_allclose(got.reshape(spec.m, spec.c_out), want, rtol=1e-5, atol=1e-6)
        dropped = got.reshape(spec.m, spec.c_out)[rm == 0]
        ref = res_dense.reshape(spec.m, spec.c_out)[rm == 0]
        assert np.array_equal(dropped, np.maximum(ref, 0.0) if post_relu else ref)     # exactly the shortcut there
        assert np.abs(dropped).max() > 0


def test_shortcut_sum_is_the_sum_of_the_two_network_ops():
    """One fused operator = conv op followed by the add / add_relu op of the network interpreter (before rounding)."""
    spec = W.ConvSpec("r", n=1, c_in=8, h=6, w=6, c_out=8, kh=1, kw=1, pad_h=0, pad_w=0, dtype="f32", relu=True, sparsity=0.5)
    x, w, b, mask = rand_inputs(spec, 73)
    res = np.random.default_rng(74).standard_normal(spec.y_shape()).astype(np.float32)
    conv = oracle.masked_conv2d(spec, x, w, b, mask)
    np.testing.assert_allclose(oracle.masked_conv2d_residual(spec, x, w, b, mask, res, True), oracle.add_relu(conv, res),
                               rtol=1e-6, atol=1e-6)
    np.testing.assert_allclose(oracle.masked_conv2d_residual(spec, x, w, b, mask, res, False), conv + res, rtol=1e-6, atol=1e-6)


def test_small_mobilenet_chain_with_masks_matches_library_pipeline():
    """Depthwise layers, linear shortcuts and 2-D masks in the network interpreter: the same graph through
    the library's grouped conv2d in float64, with the dropped pixels of every conv cleared afterwards."""
    ops = W.mobilenet_v2(batch=2, res=32, sparsity=0.5, dtype="f32")
    bs = 77
    x = W.gen_activations(W.network_input_shape(ops), bs, "f32")
    params = {}

    def layer_inputs(spec):
        if spec.name not in params:
            ci = W.make_conv_inputs(spec, bs, x=np.zeros(1, np.float32))
            params[spec.name] = (ci.w, ci.bias, ci.mask)
        return params[spec.name]

    t = oracle.run_network(ops, {"input": x}, layer_inputs)
    tt = {"input": torch.from_numpy(x).double().permute(0, 3, 1, 2)}
    for op in ops:
        if op.kind == "conv":
            s = op.spec
            w, b, m = layer_inputs(s)
            y = F.conv2d(tt[op.src], torch.from_numpy(w).double().permute(0, 3, 1, 2), torch.from_numpy(b).double(),
                         stride=s.stride_h, padding=s.pad_h, groups=s.groups)
            y = torch.relu(y) if s.relu else y
            tt[op.out] = y * torch.from_numpy(m.reshape(1, 1, s.ho, s.wo).astype(np.float64))
        else:
            assert op.kind == "add"
            tt[op.out] = tt[op.src] + tt[op.src2]
    checked = 0
    for name in ("b0_out", "b2_out", "b6_d", "b13_e", "head"):
        ref = tt[name].permute(0, 2, 3, 1).numpy()
        np.testing.assert_allclose(t[name], ref, rtol=3e-4, atol=3e-5 * max(1.0, np.abs(ref).max()))
        assert np.abs(ref).max() > 0
        checked += 1
    assert checked == 5 and t["head"].shape == (2, 1, 1, 1280)


# ---------------------------------------------------------------------------------------
# depthwise layers (groups == Cin == Cout)
# ---------------------------------------------------------------------------------------
DW_GEOMS = [
    # n, c, h, w, kh, kw, sh, sw, ph, pw, dh, dw
    (2, 5, 7, 9, 3, 3, 1, 1, 1, 1, 1, 1),
    (1, 8, 10, 6, 3, 3, 2, 2, 1, 1, 1, 1),
    (3, 3, 6, 6, 5, 5, 1, 1, 2, 2, 1, 1),
    (1, 4, 9, 8, 3, 2, 1, 2, 0, 1, 2, 1),
    (2, 6, 5, 5, 1, 1, 1, 1, 0, 0, 1, 1),
]


def dw_spec(g, bias=True, relu=False, s=0.4, mask_mode="row"):
    n, c, h, w, kh, kw, sh, sw, ph, pw, dh, dw = g
    return W.ConvSpec("dw", n=n, c_in=c, h=h, w=w, c_out=c, kh=kh, kw=kw, stride_h=sh, stride_w=sw, pad_h=ph,
                      pad_w=pw, dil_h=dh, dil_w=dw, dtype="f32", has_bias=bias, relu=relu, sparsity=s,
                      mask_mode=mask_mode, groups=c)


@pytest.mark.parametrize("g", DW_GEOMS)
@pytest.mark.parametrize("mask_mode", ["row", "spatial"])
def test_depthwise_on_compact_input_reads_zeros_at_dropped_pixels(g, mask_mode):
    """A compact input under the producer's mask is the dense map with +0.0 at the dropped pixels: the
    library's grouped conv2d on that map, masked afterwards, must agree -- also when the two masks differ
    (a strided layer reads a map of another resolution) and when both operands are compact."""
    spec = dw_spec(g, True, True, s=0.4, mask_mode=mask_mode)
    x, w, b, mask = rand_inputs(spec, 43)
    rng = np.random.default_rng(44)
    pixels = spec.h * spec.w
    x_mask = (rng.random(spec.n * pixels if mask_mode == "row" else pixels) < 0.6).astype(np.uint8)
    in_rows = x_mask if mask_mode == "row" else np.tile(x_mask, spec.n)
    xc = np.ascontiguousarray(x.reshape(-1, spec.c_in)[in_rows == 1])
    xz = x * in_rows.reshape(spec.n, spec.h, spec.w, 1)
    y = F.conv2d(torch.from_numpy(xz).double().permute(0, 3, 1, 2), torch.from_numpy(w).double().permute(0, 3, 1, 2),
                 torch.from_numpy(b).double(), stride=(spec.stride_h, spec.stride_w), padding=(spec.pad_h, spec.pad_w),
                 dilation=(spec.dil_h, spec.dil_w), groups=spec.c_in)
    rm = oracle.row_mask(spec, mask)
    ref = (torch.relu(y).permute(0, 2, 3, 1).numpy().reshape(spec.m, spec.c_out)) * rm[:, None]
    got = oracle.masked_depthwise_conv2d_compact(spec, xc, w, b, mask, x_mask=x_mask)
    np.testing.assert_allclose(got.reshape(spec.m, spec.c_out), ref, rtol=1e-5, atol=1e-6)
    assert (got.reshape(spec.m, spec.c_out)[rm == 0] == 0).all()
    got_c = oracle.masked_depthwise_conv2d_compact(spec, xc, w, b, mask, x_mask=x_mask, y_compact=True)
    np.testing.assert_allclose(got_c, ref[rm == 1], rtol=1e-5, atol=1e-6)
    # the dropped input pixels really matter: with the full map the result differs
    full = oracle.masked_depthwise_conv2d(spec, x, w, b, mask)
    if spec.kh * spec.kw > 1:
        assert not np.allclose(full.reshape(spec.m, spec.c_out), ref, rtol=1e-3, atol=1e-4)


@pytest.mark.parametrize("g", DW_GEOMS)
@pytest.mark.parametrize("bias,relu", [(False, False), (True, True)])
def test_depthwise_matches_library_grouped_conv2d(g, bias, relu):
    spec = dw_spec(g, bias, relu, s=0.0)
    x, w, b, mask = rand_inputs(spec, 41)
    assert w.shape == (spec.c_out, spec.kh, spec.kw, 1) and mask.all()
    xt = torch.from_numpy(x).double().permute(0, 3, 1, 2)
    wt = torch.from_numpy(w).double().permute(0, 3, 1, 2)
    ref = F.conv2d(xt, wt, torch.from_numpy(b).double() if bias else None, (spec.stride_h, spec.stride_w),
                   (spec.pad_h, spec.pad_w), (spec.dil_h, spec.dil_w), groups=spec.c_in)
    if relu:
        ref = torch.relu(ref)
    ref = ref.permute(0, 2, 3, 1).numpy()
    got = oracle.masked_depthwise_conv2d(spec, x, w, b, mask)
    np.testing.assert_allclose(got, ref, rtol=3e-7, atol=1e-7)
    # any mask: the dense result times the mask, exact zeros at dropped pixels
    spec_s = spec.with_(sparsity=0.4)
    mask = W.gen_mask(spec_s.mask_len, W.n_keep(0.4, spec_s.mask_len), 5)
    got = oracle.masked_depthwise_conv2d(spec_s, x, w, b, mask).reshape(spec.m, spec.c_out)
    np.testing.assert_allclose(got, ref.reshape(spec.m, spec.c_out) * mask[:, None], rtol=3e-7, atol=1e-7)
    assert (got[mask == 0].view(np.uint32) == 0).all()


@pytest.mark.parametrize("g", DW_GEOMS)
@pytest.mark.parametrize("mask_mode", ["row", "spatial"])
def test_depthwise_is_the_full_convolution_with_block_diagonal_filters(g, mask_mode):
    """A depthwise layer is an ordinary one whose filter for output channel c is zero on every other
    input channel; the ordinary oracle (pinned above) must give the same numbers."""
    spec = dw_spec(g, True, True, s=0.35, mask_mode=mask_mode)
    x, w, b, mask = rand_inputs(spec, 43)
    full = np.zeros((spec.c_out, spec.kh, spec.kw, spec.c_in), dtype=np.float32)
    for c in range(spec.c_out):
        full[c, :, :, c] = w[c, :, :, 0]
    ref, ref_abs = oracle.masked_conv2d(spec.with_(groups=1), x, full, b, mask, want_absum=True)
    got, got_abs = oracle.masked_depthwise_conv2d(spec, x, w, b, mask, want_absum=True)
    np.testing.assert_allclose(got, ref, rtol=3e-7, atol=1e-7)
    np.testing.assert_allclose(got_abs, ref_abs, rtol=1e-12, atol=1e-12)


def test_depthwise_single_tap_filters_shift_each_channel_separately():
    spec = dw_spec((1, 3, 6, 6, 3, 3, 1, 1, 1, 1, 1, 1), bias=False, relu=False, s=0.0)
    x = np.random.default_rng(47).standard_normal(spec.x_shape()).astype(np.float32)
    w = np.zeros(spec.w_shape(), np.float32)
    w[0, 1, 1, 0] = 1.0      # channel 0: centre tap, identity
    w[1, 0, 1, 0] = 2.0      # channel 1: the pixel above, doubled
    w[2, 1, 2, 0] = -1.0     # channel 2: the pixel to the right, negated
    y = oracle.masked_depthwise_conv2d(spec, x, w, None, np.ones(spec.mask_len, np.uint8))
    assert np.array_equal(y[..., 0], x[..., 0])
    assert np.array_equal(y[0, 1:, :, 1], 2.0 * x[0, :-1, :, 1]) and (y[0, 0, :, 1] == 0).all()
    assert np.array_equal(y[0, :, :-1, 2], -x[0, :, 1:, 2]) and (y[0, :, -1, 2] == 0).all()


# ---------------------------------------------------------------------------------------
# backward pass of the masked convolution (Alg. 1: backward after maskedForward)
# ---------------------------------------------------------------------------------------
def torch_masked_grads(spec, x, w, b, mask, dy):
    """Library autograd, float64: gradients of sum(dy * mask * act(conv2d(x, w) + b))."""
    xt = torch.from_numpy(x).double()
    wt = torch.from_numpy(w).double()
    if spec.layout == "nhwc":
        xt, wt = xt.permute(0, 3, 1, 2), wt.permute(0, 3, 1, 2)
    xt = xt.contiguous().requires_grad_(True)
    wt = wt.contiguous().requires_grad_(True)
    bt = torch.from_numpy(b).double().requires_grad_(True) if b is not None else None
    y = F.conv2d(xt, wt, bt, (spec.stride_h, spec.stride_w), (spec.pad_h, spec.pad_w), (spec.dil_h, spec.dil_w))
    if spec.relu:
        y = torch.relu(y)
    m = torch.from_numpy(row_mask(spec, mask).astype(np.float64)).reshape(spec.n, 1, spec.ho, spec.wo)
    y = y * m
    dyt = torch.from_numpy(dy).double()
    if spec.layout == "nhwc":
        dyt = dyt.permute(0, 3, 1, 2)
    (y * dyt).sum().backward()
    gx, gw = xt.grad, wt.grad
    if spec.layout == "nhwc":
        gx, gw = gx.permute(0, 2, 3, 1), gw.permute(0, 2, 3, 1)
    return gx.numpy(), gw.numpy(), (bt.grad.numpy() if bt is not None else None)


@pytest.mark.parametrize("g", GEOMS)
@pytest.mark.parametrize("layout", ["nhwc", "nchw"])
@pytest.mark.parametrize("relu", [False, True])
def test_backward_matches_library_autograd(g, layout, relu):
    spec = make_spec(g, layout, bias=True, relu=relu, s=0.35)
    x, w, b, mask = rand_inputs(spec, 53)
    dy = np.random.default_rng(59).standard_normal(spec.y_shape()).astype(np.float32)
    y = oracle.masked_conv2d(spec, x, w, b, mask)
    dx, dw, db = oracle.masked_conv2d_backward(spec, x, w, y, dy, mask)
    rx, rw, rb = torch_masked_grads(spec, x, w, b, mask, dy)
    np.testing.assert_allclose(dx, rx, rtol=1e-9, atol=1e-9)
    np.testing.assert_allclose(dw, rw, rtol=1e-9, atol=1e-9)
    np.testing.assert_allclose(db, rb, rtol=1e-9, atol=1e-9)


def test_backward_is_the_transposed_pipeline_on_the_kept_rows():
    """With the explicit lowering matrix A: dW = G_kept^T A_kept (fewer rows, as in the forward GEMM),
    dA_kept = G_kept W, and dx gathers dA back through the windows."""
    spec = make_spec(GEOMS[1], "nhwc", bias=True, relu=True, s=0.4)
    x, w, b, mask = rand_inputs(spec, 61)
    dy = np.random.default_rng(67).standard_normal(spec.y_shape()).astype(np.float32)
    y = oracle.masked_conv2d(spec, x, w, b, mask)
    a = lowered_matrix(spec, x)
    rm = row_mask(spec, mask)
    gmat = dy.reshape(spec.m, spec.c_out).astype(np.float64) * (y.reshape(spec.m, spec.c_out) > 0)
    gk, ak = gmat[rm == 1], a[rm == 1]
    dw_ref = (gk.T @ ak).reshape(spec.w_shape())
    da = np.zeros_like(a)
    da[rm == 1] = gk @ w.reshape(spec.c_out, spec.k).astype(np.float64)
    dx_ref = np.zeros(spec.x_shape(), np.float64)
    da = da.reshape(spec.m, spec.kh, spec.kw, spec.c_in)
    for n, oy, ox in itertools.product(range(spec.n), range(spec.ho), range(spec.wo)):
        r = (n * spec.ho + oy) * spec.wo + ox
        for ky, kx in itertools.product(range(spec.kh), range(spec.kw)):
            iy, ix = oy * spec.stride_h - spec.pad_h + ky * spec.dil_h, ox * spec.stride_w - spec.pad_w + kx * spec.dil_w
            if 0 <= iy < spec.h and 0 <= ix < spec.w:
                dx_ref[n, iy, ix, :] += da[r, ky, kx, :]
    dx, dw, db = oracle.masked_conv2d_backward(spec, x, w, y, dy, mask)
    np.testing.assert_allclose(dw, dw_ref, rtol=1e-10, atol=1e-10)
    np.testing.assert_allclose(dx, dx_ref, rtol=1e-10, atol=1e-10)
    np.testing.assert_allclose(db, gk.sum(axis=0), rtol=1e-10, atol=1e-10)


def test_backward_agrees_with_finite_differences_and_ignores_dropped_rows():
    spec = make_spec(GEOMS[0], "nhwc", bias=True, relu=False, s=0.4)
    x, w, b, mask = rand_inputs(spec, 71)
    dy = np.random.default_rng(73).standard_normal(spec.y_shape()).astype(np.float32)
    y = oracle.masked_conv2d(spec, x, w, b, mask)
    dx, dw, db = oracle.masked_conv2d_backward(spec, x, w, y, dy, mask)
    loss = lambda xx, ww: float((oracle.masked_conv2d(spec, xx, ww, b, mask).astype(np.float64) * dy).sum())
    eps = 1e-2      # the layer is linear without the ReLU: a central difference is exact up to rounding
    for idx in [(0, 2, 3, 1), (0, 0, 0, 0), (0, 4, 4, 2)]:
        xp, xm = x.copy(), x.copy()
        xp[idx] += eps
        xm[idx] -= eps
        assert abs((loss(xp, w) - loss(xm, w)) / (2 * eps) - dx[idx]) < 1e-3
    for idx in [(1, 0, 2, 1), (0, 1, 1, 0)]:
        wp, wm = w.copy(), w.copy()
        wp[idx] += eps
        wm[idx] -= eps
        assert abs((loss(x, wp) - loss(x, wm)) / (2 * eps) - dw[idx]) < 1e-3
    # the upstream gradient of a dropped row changes nothing
    dy2 = dy.copy().reshape(spec.m, spec.c_out)
    dy2[mask == 0] = 1e6
    dx2, dw2, db2 = oracle.masked_conv2d_backward(spec, x, w, y, dy2.reshape(spec.y_shape()), mask)
    assert np.array_equal(dx2, dx) and np.array_equal(dw2, dw) and np.array_equal(db2, db)
