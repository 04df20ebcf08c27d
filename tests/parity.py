"""Shared helpers of the GPU parity tests: run one layer through the C ABI and compare it with
the CPU oracle element by element."""
import numpy as np
import torch

import workloads as W
from oracle import oracle
from paper_2309_06626_amd import binding as B
from paper_2309_06626_amd import runtime as R

# tolerances: 1e-5 (fp32) and 2e-2 (bf16) relative, as the targets of this build state; fp16
# keeps 11 significant bits (output rounding 2^-11), so it gets a tighter bound than bf16.
TOL = {"f32": 1e-5, "bf16": 2e-2, "f16": 4e-3}


def rows_view(spec, y):
    """[M, Cout] view of a host array in the layer's output layout."""
    if spec.layout == "nchw":
        y = np.transpose(y, (0, 2, 3, 1))
    return np.ascontiguousarray(y).reshape(spec.m, spec.c_out)


def row_mask(spec, mask):
    return np.tile(mask, spec.n) if spec.mask_mode == "spatial" else mask


def assert_close(got, ref, absum, tol, what=""):
    """got/ref: float arrays of equal shape (kept rows); absum: sum|x*w|+|bias| per element.

    (i) normwise, (ii) max error against the largest reference magnitude, (iii) per element
    against the magnitude of the summed terms -- relative error proper is undefined at the
    exact zeros a ReLU produces."""
    got = got.astype(np.float64)
    ref = ref.astype(np.float64)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    if ref.size == 0:
        return
    err = np.abs(got - ref)
    nref = np.linalg.norm(ref)
    if nref > 0:
        assert np.linalg.norm(got - ref) / nref <= tol, f"{what}: normwise {np.linalg.norm(got - ref) / nref:.3e}"
    mref = np.abs(ref).max()
    if mref > 0:
        assert err.max() / mref <= tol, f"{what}: max error {err.max() / mref:.3e}"
    bound = tol * absum + 1e-30
    worst = (err / bound).max()
    assert worst <= 1.0, f"{what}: element error is {worst:.3f} x the allowed tol*sum|x*w|"


def check_layer(ci: W.ConvInputs, tiles=None, out_mode=B.SC_OUT_ZERO_FILL, check_dense=True, sample_rows=None,
                device="cuda:0", check_count=True, split_k=None, row_panel=None, stream_k=None, options=None):
    """Plan + sparse run (+ dense run) of one layer, compared with the oracle.

    sample_rows: None = every row through the oracle, else that many random rows plus every
    structural check (dropped rows zero, kept rows finite) on the whole output."""
    spec = ci.spec
    tol = TOL[spec.dtype]
    layer = R.ConvLayer(spec, ci.w, ci.bias, ci.mask, device=device, out_mode=out_mode, check_count=check_count)
    if tiles is not None:   # (tile_m, tile_n) of the tiled kernel, or (-1, 0) for the band kernel
        B.sparse_conv_plan_set_tiles(layer.plan, 0, *tiles)
        B.sparse_conv_plan_set_tiles(layer.plan, 1, *tiles)
    if split_k is not None:
        B.sparse_conv_plan_set_option(layer.plan, B.SC_OPT_SPLIT_K, split_k)
    if row_panel is not None:
        B.sparse_conv_plan_set_option(layer.plan, B.SC_OPT_ROW_PANEL, row_panel)
    if stream_k is not None:
        B.sparse_conv_plan_set_option(layer.plan, B.SC_OPT_STREAM_K, stream_k)
    for option, value in (options or {}).items():
        B.sparse_conv_plan_set_option(layer.plan, option, value)
    rm = row_mask(spec, ci.mask)

    # a0: compaction, bit-exact
    want_rows = oracle.compact_rows(rm)
    info = layer.info
    assert info["m"] == spec.m and info["ho"] == spec.ho and info["wo"] == spec.wo
    assert info["kept"] == want_rows.size
    got_rows = B.plan_row_idx(layer.plan).cpu().numpy()
    assert got_rows.dtype == np.int32 and np.array_equal(got_rows, want_rows)

    x = R.to_device(ci.x, spec.dtype, device)
    sentinel = float("nan") if out_mode == B.SC_OUT_ZERO_FILL else 7.0
    y = layer.new_output()
    y.fill_(sentinel)
    layer.sparse(x, y)
    torch.cuda.synchronize()
    bits = rows_view(spec, R.bits_of(y))
    g = rows_view(spec, R.to_host_f32(y))
    kept = rm == 1

    # dropped rows: exact zeros (or untouched in scatter-only mode)
    if out_mode == B.SC_OUT_ZERO_FILL:
        assert (bits[~kept] == 0).all(), "dropped rows must be +0.0 in every channel"
    else:
        assert (g[~kept] == 7.0).all(), "scatter-only mode must not touch dropped rows"
    assert np.isfinite(g[kept]).all()

    # determinism
    y2 = layer.new_output()
    y2.fill_(sentinel)
    layer.sparse(x, y2)
    torch.cuda.synchronize()
    assert np.array_equal(R.bits_of(y2), R.bits_of(y)), "two runs differ"

    if sample_rows is None:
        ref, absum = oracle.masked_conv2d(spec, ci.x, ci.w, ci.bias, ci.mask, want_absum=True)
        ref, absum = rows_view(spec, ref), rows_view(spec, absum)
        assert_close(g[kept], ref[kept], absum[kept], tol, f"{spec.name} sparse")
        sel = None
    else:
        rng = np.random.default_rng(1234)
        sel = np.unique(np.concatenate([rng.integers(0, spec.m, sample_rows), [0, spec.m - 1]])).astype(np.int64)
        ref_s, absum_s = oracle.masked_conv2d_rows(spec, ci.x, ci.w, ci.bias, ci.mask, sel, want_absum=True)
        ks = kept[sel]
        assert_close(g[sel][ks], ref_s[ks], absum_s[ks], tol, f"{spec.name} sparse (sampled)")
        assert (ref_s[~ks] == 0).all()

    if check_dense:
        yd = layer.new_output()
        yd.fill_(float("nan"))
        layer.dense(x, yd)
        torch.cuda.synchronize()
        gd = rows_view(spec, R.to_host_f32(yd))
        ones = np.ones_like(ci.mask)
        if sample_rows is None:
            refd, absd = oracle.masked_conv2d(spec, ci.x, ci.w, ci.bias, ones, want_absum=True)
            assert_close(gd, rows_view(spec, refd), rows_view(spec, absd), tol, f"{spec.name} dense")
        else:
            refd, absd = oracle.masked_conv2d_rows(spec, ci.x, ci.w, ci.bias, ones, sel, want_absum=True)
            assert_close(gd[sel], refd, absd, tol, f"{spec.name} dense (sampled)")
        # sparse kept rows against the dense run of the same kernels
        assert_close(g[kept], gd[kept], np.abs(gd[kept]).astype(np.float64) + 1e-3, 2 * tol, f"{spec.name} sparse~dense")
    return layer


def compare_network(ops, dev, ref, params, tol, absums=None):
    """Every tensor of a network run against the oracle's: normwise, against the largest reference magnitude, and --
    with `absums` from the oracle's interpreter -- element by element against tol * (sum |x*w| + |bias|) of the
    convolution that produced it, the bound check_layer applies to single layers.  (Both sides feed every layer with
    their own rounded previous outputs, so an element's error also carries what its inputs differed by; the bound
    is the same one all the same.)"""
    for op in ops:
        g, r = R.to_host_f32(dev[op.out]), ref[op.out]
        assert g.shape == r.shape
        nr = np.linalg.norm(r.astype(np.float64))
        err = np.linalg.norm(g.astype(np.float64) - r.astype(np.float64)) / max(nr, 1e-30)
        assert err <= tol, f"{op.out}: normwise {err:.3e}"
        assert np.abs(g - r).max() <= tol * max(np.abs(r).max(), 1e-30), op.out
        if absums is not None and op.kind == "conv":
            bound = tol * absums[op.out].reshape(r.shape) + 1e-30
            worst = (np.abs(g.astype(np.float64) - r) / bound).max()
            assert worst <= 1.0, f"{op.out}: element error is {worst:.3f} x the allowed tol*sum|x*w|"
        if op.kind == "conv":
            mask = params[op.spec.name][2]
            bits = rows_view(op.spec, R.bits_of(dev[op.out]))
            assert (bits[mask == 0] == 0).all(), f"{op.out}: dropped rows must be zero"
