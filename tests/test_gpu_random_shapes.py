"""Seeded random layer shapes through the HIP path against the oracle: every kernel family, forced tile shapes,
stream-K launches, fused shortcut sums, depthwise layers and compact depthwise inputs.  The samplers draw what the
hand-written cases fix by hand -- window, stride, padding, dilation, channel counts with and without 16-byte groups,
layouts, dtypes, mask modes, sparsities, output modes -- so that ragged tiles and odd combinations nobody listed are
covered too.  Each case prints itself first: a failure names its shape."""
import random

import pytest

import workloads as W
from paper_2309_06626_amd import binding as B
from parity import check_layer
from test_gpu_depthwise import check_compact_input, check_depthwise, dw_spec
from test_gpu_parity import spec_of
from test_gpu_residual import check as check_residual

pytestmark = pytest.mark.gpu

TILES = [None, (128, 128), (128, 64), (96, 128), (64, 128), (64, 64), (128, 32), (32, 128)]


def _smallest(k, d, p):
    return max(5, d * (k - 1) + 2 - 2 * p)


@pytest.mark.parametrize("seed", [7, 11, 23])
def test_random_deep_layers_with_forced_tiles_stream_k_and_shortcuts(seed):
    """Input channels in multiples of 64 (the buffer-load tiled kernel), every tile shape, stream-K where it applies."""
    rnd = random.Random(seed)
    for it in range(40):
        k = rnd.choice([1, 3, 3, 3, 5]); s = rnd.choice([1, 1, 2]); d = rnd.choice([1, 1, 2]) if k > 1 else 1
        p = rnd.randint(0, (k // 2) * d + (1 if k > 1 else 0))
        cin = rnd.choice([64, 64, 128, 192, 256, 512]); cout = 16 * rnd.randint(1, 20)
        h, w = rnd.randint(_smallest(k, d, p), 22), rnd.randint(_smallest(k, d, p), 22)
        n = rnd.randint(1, 4); sp = rnd.choice([0.0, 0.3, 0.5, 0.5, 0.7, 0.9])
        dtype = rnd.choice(["bf16", "f16"]); mm = rnd.choice(["row", "spatial"])
        tile = rnd.choice(TILES)
        spec = spec_of(n, cin, h, w, cout, k=k, s=s, p=p, d=d, dtype=dtype, sp=sp, mask_mode=mm, relu=rnd.choice([True, False]))
        splittable = tile in [(128, 128), (128, 64), (64, 128), (64, 64)] and spec.k // 64 >= 16 and cout >= 128
        sk = rnd.choice([None, None, 8, 24]) if splittable else None
        fused = tile is None and sk is None and rnd.random() < 0.34
        post = rnd.choice([True, False])
        print(f"seed {seed} case {it}: {spec} tile={tile} stream_k={sk} fused={fused}", flush=True)
        if fused:
            check_residual(spec, 5000 + 100 * seed + it, post)
        else:
            check_layer(W.make_conv_inputs(spec, 5000 + 100 * seed + it), tiles=tile, stream_k=sk)


@pytest.mark.parametrize("seed", [3, 17, 29])
def test_random_layers_with_the_automatic_kernel_choice(seed):
    """Any channel counts, layouts and dtypes with the kernel the plan picks, plus depthwise layers with dense and compact inputs."""
    rnd = random.Random(seed)
    for it in range(60):
        kind = rnd.choice(["conv", "conv", "conv", "dw", "dwc"])
        if kind == "conv":
            k = rnd.choice([1, 1, 3, 3, 3, 5, 7]); s = rnd.choice([1, 1, 2]); d = rnd.choice([1, 1, 1, 2]) if k > 1 else 1
            p = rnd.randint(0, (k // 2) * d + (1 if k > 1 else 0))
            cin = rnd.choice([3, 8, 16, 16, 19, 24, 32, 32, 48, 64, 64, 96, 128, 144, 192])
            cout = rnd.choice([8, 16, 21, 32, 32, 48, 64, 64, 96, 128, 160, 192, 320, 576])
            lo = max(4, d * (k - 1) + 2 - 2 * p)
            h, w, n = rnd.randint(lo, 40), rnd.randint(lo, 40), rnd.randint(1, 6)
            dtype = rnd.choice(["bf16", "bf16", "f16", "f32"]); layout = rnd.choice(["nhwc", "nhwc", "nhwc", "nchw"])
            sp = rnd.choice([0.0, 0.25, 0.5, 0.5, 0.7, 0.95]); mm = rnd.choice(["row", "spatial"])
            om = rnd.choice([B.SC_OUT_ZERO_FILL, B.SC_OUT_ZERO_FILL, B.SC_OUT_SCATTER_ONLY])
            spec = spec_of(n, cin, h, w, cout, k=k, s=s, p=p, d=d, dtype=dtype, layout=layout, sp=sp, mask_mode=mm,
                           relu=rnd.choice([True, False]), bias=rnd.choice([True, True, False]))
            print(f"seed {seed} case {it}: {spec} out_mode={om}", flush=True)
            check_layer(W.make_conv_inputs(spec, 7000 + 100 * seed + it), out_mode=om)
        else:
            c = rnd.choice([8, 16, 24, 32, 40, 96, 144, 192]); k = rnd.choice([3, 3, 3, 5]); s = rnd.choice([1, 2])
            h, w, n = rnd.randint(6, 40), rnd.randint(6, 40), rnd.randint(1, 5)
            dtype = rnd.choice(["bf16", "f16", "f32"]) if kind == "dw" else rnd.choice(["bf16", "f16"])
            spec = dw_spec(n, c, h, w, k=k, s=s, dtype=dtype, sparsity=rnd.choice([0.0, 0.3, 0.5, 0.8]),
                           mask_mode=rnd.choice(["row", "spatial"]))
            print(f"seed {seed} case {it}: {kind} {spec}", flush=True)
            if kind == "dw":
                check_depthwise(spec, 7000 + 100 * seed + it, rnd.choice([B.SC_OUT_ZERO_FILL, B.SC_OUT_SCATTER_ONLY]))
            else:
                check_compact_input(spec, 7000 + 100 * seed + it, in_sparsity=rnd.choice([0.0, 0.4, 0.6]))


@pytest.mark.parametrize("seed", [5, 13])
def test_random_backward_passes_compact_outputs_and_generated_masks(seed):
    """The widened rows under the same treatment: gradients (strides 1-3, dilation, ragged channel counts in multiples of 8),
    compact outputs of pointwise and 3x3 layers, and masks from random scores (tie-heavy ones among them)."""
    import numpy as np

    import test_gpu_backward as TB
    import test_gpu_compact as TC
    import test_gpu_mask as TM
    from oracle import mask_oracle as MO

    rnd = random.Random(seed)
    for it in range(45):
        kind = rnd.choice(["bwd", "bwd", "compact", "mask"])
        if kind == "bwd":
            k = rnd.choice([1, 3, 3, 5]); s = rnd.choice([1, 1, 2, 3]); d = rnd.choice([1, 1, 2]) if k > 1 else 1
            cin, cout = 8 * rnd.randint(1, 20), 8 * rnd.randint(1, 24)
            lo = max(5, d * (k - 1) + 1)
            spec = TB.spec_of(rnd.randint(1, 4), cin, rnd.randint(lo, 24), cout, k=k, s=s, d=d, dtype=rnd.choice(["bf16", "f16"]),
                              sparsity=rnd.choice([0.0, 0.3, 0.5, 0.8]), relu=rnd.choice([True, False]),
                              mask_mode=rnd.choice(["row", "spatial"]), w=rnd.randint(lo, 24))
            print(f"seed {seed} case {it}: backward {spec}", flush=True)
            TB.run_backward(spec, 9000 + 100 * seed + it)
        elif kind == "compact":
            k = rnd.choice([1, 1, 3, 3])
            cin = rnd.choice([8, 16, 32, 48, 64, 96, 128, 192, 256]); cout = rnd.choice([16, 32, 48, 64, 96, 128, 160, 192, 576])
            spec = TC.layer_spec("c", rnd.randint(1, 5), cin, rnd.randint(5, 30), cout, k=k, s=rnd.choice([1, 1, 2]),
                                 dtype=rnd.choice(["bf16", "f16", "f32"]), sparsity=rnd.choice([0.0, 0.3, 0.5, 0.9]),
                                 mask_mode=rnd.choice(["row", "spatial"]), w=rnd.randint(5, 30))
            print(f"seed {seed} case {it}: compact output {spec}", flush=True)
            TC.check_compact_output(spec, 9000 + 100 * seed + it)
        else:
            ho, wo = rnd.randint(1, 90), rnd.randint(1, 90)
            ry, rx = rnd.choice([1, 1, 2, 3, 4, 8]), rnd.choice([1, 1, 2, 3, 4, 8])
            h, w = ho * ry + rnd.randint(0, ry - 1), wo * rx + rnd.randint(0, rx - 1)
            s = rnd.choice([0.0, 0.1, 0.25, 0.5, 0.7, 0.93, 1.0])
            score = W.gen_score(h, w, seed=9000 + 100 * seed + it)
            if rnd.random() < 0.3:
                score = np.round(score * rnd.choice([2, 5, 17])).astype(np.float32)     # a handful of levels: ties everywhere
            print(f"seed {seed} case {it}: mask {h}x{w} -> {ho}x{wo} s={s}", flush=True)
            assert np.array_equal(TM.gpu_mask(score, ho, wo, s), MO.layer_mask(score, ho, wo, TM.f32(s)))
