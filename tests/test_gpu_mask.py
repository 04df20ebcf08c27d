"""Mask generator (Alg. 1, getMask) on the GPU against its CPU oracle, through the C ABI: masks are
bytes, so every comparison is bit-exact."""
import numpy as np
import pytest
import torch

import paper_2309_06626_amd.binding as B
import paper_2309_06626_amd.runtime as R
import workloads as W
from oracle import mask_oracle as MO
from oracle import oracle
from parity import TOL, compare_network

pytestmark = pytest.mark.gpu


def f32(s):
    """The sparsity as the C ABI receives it (a float)."""
    return float(np.float32(s))


def gpu_mask(score, ho, wo, s):
    dev = torch.from_numpy(score).to("cuda:0")
    mask = torch.full((ho, wo), 7, dtype=torch.uint8, device="cuda:0")      # poison: every byte must be written
    B.sparse_mask_generate(dev, ho, wo, s, mask=mask)
    torch.cuda.synchronize()
    return mask.cpu().numpy()


@pytest.mark.parametrize("h,w,ho,wo", [
    (224, 224, 112, 112), (224, 224, 56, 56), (224, 224, 28, 28), (224, 224, 14, 14), (224, 224, 7, 7),
    (64, 64, 64, 64), (33, 47, 16, 15), (9, 9, 4, 4), (15, 10, 7, 3), (5, 3, 1, 1), (1, 1, 1, 1), (640, 640, 80, 80),
    (640, 640, 320, 320), (640, 640, 20, 20), (300, 270, 10, 9), (100, 100, 2, 2), (70, 70, 1, 1), (130, 129, 128, 129),
    (200, 300, 200, 150),
])
@pytest.mark.parametrize("s", [0.25, 0.5, 0.7])
def test_masks_match_the_oracle(h, w, ho, wo, s):
    score = W.gen_score(h, w, seed=h * 1000 + ho)
    want = MO.layer_mask(score, ho, wo, f32(s))
    got = gpu_mask(score, ho, wo, s)
    assert got.shape == want.shape and np.array_equal(got, want)
    assert int(got.sum()) == MO.kept_pixels(f32(s), ho * wo)


@pytest.mark.parametrize("s", [0.0, 1.0, 0.001, 0.999])
def test_extreme_sparsities(s):
    score = W.gen_score(48, 48, seed=3)
    for ho in (48, 12):
        assert np.array_equal(gpu_mask(score, ho, ho, s), MO.layer_mask(score, ho, ho, f32(s)))


@pytest.mark.parametrize("levels", [1, 2, 3, 40])
def test_ties_are_dropped_in_index_order(levels):
    """Few distinct score values: the selected key is shared by many pixels, which go by index."""
    rng = np.random.default_rng(levels)
    score = rng.integers(0, levels, size=(96, 80)).astype(np.float32)
    for (ho, wo), s in [((96, 80), 0.5), ((96, 80), 0.31), ((48, 40), 0.5), ((12, 10), 0.7)]:
        assert np.array_equal(gpu_mask(score, ho, wo, s), MO.layer_mask(score, ho, wo, f32(s)))


def test_negative_scores_zero_signs_and_infinities():
    rng = np.random.default_rng(8)
    score = rng.standard_normal((40, 40)).astype(np.float32)
    score[rng.random((40, 40)) < 0.2] = 0.0
    score[rng.random((40, 40)) < 0.1] = -0.0
    score[3, 3], score[20, 7] = np.inf, -np.inf
    for ho, s in [(40, 0.5), (40, 0.25), (20, 0.5), (10, 0.6)]:
        assert np.array_equal(gpu_mask(score, ho, ho, s), MO.layer_mask(score, ho, ho, f32(s)))


@pytest.mark.parametrize("levels", [1, 2, 5, 3000, 200000])
def test_ties_on_a_large_map(levels):
    """More than 16 384 pixels (the selection spread over many workgroups): one key for the whole map, a few keys shared
    by more pixels than the candidate list holds (the last workgroup selects from memory), and many keys that each
    a handful of pixels share (ties inside the candidate list)."""
    rng = np.random.default_rng(levels)
    score = rng.integers(0, levels, size=(180, 160)).astype(np.float32)
    for (ho, wo), s in [((180, 160), 0.5), ((180, 160), 0.31), ((180, 160), 0.002), ((90, 160), 0.7)]:
        assert np.array_equal(gpu_mask(score, ho, wo, s), MO.layer_mask(score, ho, wo, f32(s))), (ho, wo, s)


def test_keys_of_both_signs_and_infinities_on_a_large_map():
    rng = np.random.default_rng(81)
    score = rng.standard_normal((200, 200)).astype(np.float32)
    score[rng.random((200, 200)) < 0.1] = 0.0
    score[5, 5], score[100, 7], score[199, 199] = np.inf, -np.inf, np.inf
    for ho, s in [(200, 0.5), (200, 0.9)]:
        assert np.array_equal(gpu_mask(score, ho, ho, s), MO.layer_mask(score, ho, ho, f32(s)))


@pytest.mark.parametrize("h,w,ho,wo", [(256, 256, 8, 8), (70, 70, 1, 1), (100, 100, 2, 2), (640, 640, 20, 20), (640, 320, 40, 10)])
def test_large_windows_whose_sums_round(h, w, ho, wo):
    """Windows of 64 values and more with magnitudes spread over forty binades: additions round, so only the
    row-major chain gives the oracle's sums (scores on a 2^-24 grid never get there: their sums are exact in any order)."""
    rng = np.random.default_rng(h + wo)
    score = (rng.standard_normal((h, w)) * 10.0 ** rng.uniform(-9, 3, size=(h, w))).astype(np.float32)
    for s in (0.5, 0.3):
        assert np.array_equal(gpu_mask(score, ho, wo, s), MO.layer_mask(score, ho, wo, f32(s)))


def test_a_window_that_stops_being_exact_in_a_later_piece():
    """50 x 50 windows arrive in pieces; a tiny value late in one window makes that pixel switch to the chain."""
    score = W.gen_score(100, 100, seed=77)
    score[45, 10] = np.float32(1e-30)
    score[97, 60] = np.float32(-3e-33)
    for s in (0.5, 0.25, 0.75):
        assert np.array_equal(gpu_mask(score, 2, 2, s), MO.layer_mask(score, 2, 2, f32(s)))


@pytest.mark.parametrize("ho,win", [(8, 32), (4, 50), (12, 8), (16, 5)])
def test_windows_that_hold_the_same_values_in_different_orders(ho, win):
    """Every window is a permutation of one set of values spread over forty binades: the exact sums are equal, the
    sums in double differ only by where the additions rounded, so the ranking follows the order of the additions --
    any order but the row-major one gives another mask."""
    rng = np.random.default_rng(ho * win)
    base = (rng.standard_normal(win * win) * 10.0 ** rng.uniform(-9, 3, size=win * win)).astype(np.float32)
    score = np.empty((ho * win, ho * win), dtype=np.float32)
    for oy in range(ho):
        for ox in range(ho):
            score[oy * win:(oy + 1) * win, ox * win:(ox + 1) * win] = rng.permutation(base).reshape(win, win)
    sums = MO.layer_score_sums(score, ho, ho)
    assert len(np.unique(sums)) >= 3                     # the orders do round differently
    for s in (0.5, 0.3):
        assert np.array_equal(gpu_mask(score, ho, ho, s), MO.layer_mask(score, ho, ho, f32(s)))
    grid = np.round(score.astype(np.float64) * 2.0 ** 10).astype(np.float32)      # same idea where no addition rounds
    grid = np.clip(grid, -2.0 ** 20, 2.0 ** 20)
    assert len(np.unique(MO.layer_score_sums(grid, ho, ho))) == 1
    assert np.array_equal(gpu_mask(grid, ho, ho, 0.4), MO.layer_mask(grid, ho, ho, f32(0.4)))


def test_large_map_with_narrow_score_range():
    """All sums share their leading digits, so the first radix passes cannot shrink the candidate set."""
    rng = np.random.default_rng(12)
    score = (1.0 + rng.random((320, 320), dtype=np.float32) * np.float32(1e-3)).astype(np.float32)
    for ho, s in [(320, 0.5), (160, 0.3)]:
        assert np.array_equal(gpu_mask(score, ho, ho, s), MO.layer_mask(score, ho, ho, f32(s)))


def test_resnet_stack_with_propagated_masks():
    """Alg. 1 end to end on the inference side: one score, one mask per layer resolution from the GPU
    generator, fed as 2-D masks to every convolution of the ResNet18 stack; the oracle does the same
    with its own masks."""
    ops = W.with_spatial_masks(W.config3(batch=2))
    bs = W.base_seed(3)
    res = W.network_input_shape(ops)[1]
    score = W.gen_score(res, res, seed=bs + 77)
    score_dev = torch.from_numpy(score).to("cuda:0")
    params = {}
    masks_dev = {}
    for spec in W.conv_specs(ops):
        ci = W.make_conv_inputs(spec, bs, x=np.zeros(1, np.float32))
        want = MO.layer_mask(score, spec.ho, spec.wo, f32(spec.sparsity)).reshape(-1)
        got = B.sparse_mask_generate(score_dev, spec.ho, spec.wo, spec.sparsity)
        torch.cuda.synchronize()
        assert np.array_equal(got.cpu().numpy().reshape(-1), want), spec.name
        params[spec.name] = (ci.w, ci.bias, want)
        masks_dev[spec.name] = got
    # layers at one resolution share one mask (the propagation property)
    assert np.array_equal(params["l1b0_conv1"][2], params["l1b1_conv2"][2])
    dtype = "bf16"
    host = {"input": W.gen_activations(W.network_input_shape(ops), bs, dtype)}
    layers = {s.name: R.ConvLayer(s, params[s.name][0], params[s.name][1], masks_dev[s.name].cpu().numpy().reshape(-1))
              for s in W.conv_specs(ops)}
    dev = R.run_network(ops, {k: R.to_device(v, dtype) for k, v in host.items()}, layers)
    torch.cuda.synchronize()
    ref = oracle.run_network(ops, host, lambda spec: params[spec.name])
    row_params = {k: (v[0], v[1], np.tile(v[2], 2)) for k, v in params.items()}     # per-row masks for the zero check
    compare_network(ops, dev, ref, row_params, TOL["bf16"])


def test_training_style_steps_refresh_mask_and_filters_of_one_plan():
    """Alg. 1, main loop: every step draws a new score, getMask turns it into the layer's mask, the optimiser
    has changed the weights, and the same plan runs the masked forward pass with both."""
    spec = W.ConvSpec("train", n=3, c_in=32, h=28, w=28, c_out=64, dtype="bf16", sparsity=0.5, mask_mode="spatial")
    ci = W.make_conv_inputs(spec, 601)
    layer = R.ConvLayer(spec, ci.w, ci.bias, ci.mask)
    x = R.to_device(ci.x, spec.dtype)
    rng = np.random.default_rng(607)
    seen = []
    for step in range(4):
        score = W.gen_score(224, 224, seed=700 + step)
        mask_dev = B.sparse_mask_generate(torch.from_numpy(score).to("cuda:0"), spec.ho, spec.wo, spec.sparsity)
        w_step = W.quantize(ci.w + np.float32(0.01) * rng.standard_normal(ci.w.shape).astype(np.float32), spec.dtype)
        B.sparse_conv_plan_set_mask(layer.plan, mask_dev)
        B.sparse_conv_plan_set_filters(layer.plan, R.to_device(w_step, spec.dtype))
        mask = MO.layer_mask(score, spec.ho, spec.wo, f32(spec.sparsity)).reshape(-1)
        assert np.array_equal(mask_dev.cpu().numpy().reshape(-1), mask)
        seen.append(mask)
        rm = np.tile(mask, spec.n)
        assert np.array_equal(B.plan_row_idx(layer.plan).cpu().numpy(), oracle.compact_rows(rm))
        y = layer.new_output(fill_nan=True)
        layer.sparse(x, y)
        torch.cuda.synchronize()
        ref, absum = oracle.masked_conv2d(spec, ci.x, w_step, ci.bias, mask, want_absum=True)
        from parity import assert_close, rows_view
        g, bits = rows_view(spec, R.to_host_f32(y)), rows_view(spec, R.bits_of(y))
        assert (bits[rm == 0] == 0).all()
        assert_close(g[rm == 1], rows_view(spec, ref)[rm == 1], rows_view(spec, absum)[rm == 1], TOL["bf16"], f"step {step}")
    assert not np.array_equal(seen[0], seen[1])      # the masks really changed between steps
    # a mask with the wrong count is refused; a good one afterwards puts the plan back to work
    bad = torch.ones(spec.ho * spec.wo, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(B.ScError):
        B.sparse_conv_plan_set_mask(layer.plan, bad)
    B.sparse_conv_plan_set_mask(layer.plan, torch.from_numpy(seen[0]).to("cuda:0"))
    y = layer.new_output(fill_nan=True)
    layer.sparse(x, y)
    torch.cuda.synchronize()
    assert (rows_view(spec, R.bits_of(y))[np.tile(seen[0], spec.n) == 0] == 0).all()
