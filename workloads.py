"""Seeded synthetic workloads: layer shapes and input tensors.

This module is shared by the tests, the benchmark and the smoke check.  It holds
only *descriptions* (layer shapes, network wiring) and *random input
generators*; none of the masked-convolution arithmetic lives here, and it
imports neither the HIP binding nor the CPU oracle.

The shapes stand in for the networks the paper evaluates (ResNet18,
MobileNetV2, a YOLO-style detector; Sec. 4.1) -- only their per-layer
Cin/Cout/H/W are taken, never data or weights.  The value distributions are:

* activations  x = max(N(0,1), 0)          (post-ReLU half-normal, half zeros)
* weights      w = N(0, 2 / (Cin*kh*kw))   (Kaiming-normal, fan-in)
* bias         b = N(0, 0.1^2)
* row mask     exactly ``kept`` ones, the dropped positions drawn uniformly
               without replacement (Sec. 3: the sparsity is unstructured over
               the spatial positions and removes all channels of a position).

Every tensor has its own seed: ``base_seed + 1000*layer + {0:x,1:w,2:bias,3:mask}``
with ``base_seed = 2309 + config index``.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, replace
from typing import Dict, List, Optional

import numpy as np

# --------------------------------------------------------------------------------------
# dtype helpers (storage encodings only)
# --------------------------------------------------------------------------------------

DTYPES = ("f32", "f16", "bf16")


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even) and return the uint16 patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns exactly to float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def quantize(a: np.ndarray, dtype: str) -> np.ndarray:
    """Return ``a`` rounded once to ``dtype`` and widened back to float32 (exact)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "f32":
        return a
    if dtype == "f16":
        return a.astype(np.float16).astype(np.float32)
    if dtype == "bf16":
        return bf16_bits_to_f32(f32_to_bf16_bits(a))
    raise ValueError(dtype)


def encode(a: np.ndarray, dtype: str) -> np.ndarray:
    """Storage encoding of already-representable float32 values.

    f32 -> float32, f16 -> float16, bf16 -> uint16 bit patterns.
    """
    if dtype == "f32":
        return np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "f16":
        return np.ascontiguousarray(a, dtype=np.float32).astype(np.float16)
    if dtype == "bf16":
        return f32_to_bf16_bits(a)
    raise ValueError(dtype)


def decode(a: np.ndarray, dtype: str) -> np.ndarray:
    """Inverse of :func:`encode` (exact widening to float32)."""
    if dtype == "f32":
        return np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "f16":
        return np.ascontiguousarray(a).view(np.float16).astype(np.float32)
    if dtype == "bf16":
        return bf16_bits_to_f32(np.ascontiguousarray(a).view(np.uint16))
    raise ValueError(dtype)


# --------------------------------------------------------------------------------------
# layer description
# --------------------------------------------------------------------------------------


@dataclass(frozen=True)
class ConvSpec:
    """One convolution layer and its row mask recipe."""

    name: str
    n: int
    c_in: int
    h: int
    w: int
    c_out: int
    kh: int = 3
    kw: int = 3
    stride_h: int = 1
    stride_w: int = 1
    pad_h: int = 1
    pad_w: int = 1
    dil_h: int = 1
    dil_w: int = 1
    dtype: str = "bf16"
    layout: str = "nhwc"  # "nhwc": x[N,H,W,C], w[O,kh,kw,I]; "nchw": x[N,C,H,W], w[O,I,kh,kw]
    has_bias: bool = True
    relu: bool = True
    sparsity: float = 0.5
    mask_mode: str = "row"  # "row": uint8[N*Ho*Wo]; "spatial": uint8[Ho*Wo] shared by the batch
    layer_index: int = 0
    groups: int = 1  # 1, or c_in == c_out == groups: depthwise (every channel has its own kh x kw filter)

    @property
    def ho(self) -> int:
        return (self.h + 2 * self.pad_h - self.dil_h * (self.kh - 1) - 1) // self.stride_h + 1

    @property
    def wo(self) -> int:
        return (self.w + 2 * self.pad_w - self.dil_w * (self.kw - 1) - 1) // self.stride_w + 1

    @property
    def m(self) -> int:
        return self.n * self.ho * self.wo

    @property
    def k(self) -> int:
        return self.kh * self.kw * (self.c_in // self.groups)

    @property
    def mask_len(self) -> int:
        return self.m if self.mask_mode == "row" else self.ho * self.wo

    def x_shape(self):
        return (self.n, self.h, self.w, self.c_in) if self.layout == "nhwc" else (self.n, self.c_in, self.h, self.w)

    def w_shape(self):
        if self.layout == "nhwc":
            return (self.c_out, self.kh, self.kw, self.c_in // self.groups)
        return (self.c_out, self.c_in // self.groups, self.kh, self.kw)

    def y_shape(self):
        if self.layout == "nhwc":
            return (self.n, self.ho, self.wo, self.c_out)
        return (self.n, self.c_out, self.ho, self.wo)

    def with_(self, **kw) -> "ConvSpec":
        return replace(self, **kw)


def n_keep(sparsity: float, positions: int) -> int:
    """Number of ones in a workload mask: the mask recipe drops the fraction
    ``sparsity`` of the positions, rounded half up (never Python's banker's round)."""
    return int(math.floor((1.0 - float(sparsity)) * positions + 0.5))


# --------------------------------------------------------------------------------------
# tensor generators
# --------------------------------------------------------------------------------------


def _seed(base_seed: int, layer: int, which: int) -> int:
    return int(base_seed) + 1000 * int(layer) + int(which)


def gen_activations(shape, seed: int, dtype: str) -> np.ndarray:
    rng = np.random.default_rng(seed)
    x = np.maximum(rng.standard_normal(size=shape, dtype=np.float32), np.float32(0.0))
    return quantize(x, dtype)


def gen_weights(spec: ConvSpec, seed: int) -> np.ndarray:
    rng = np.random.default_rng(seed)
    std = math.sqrt(2.0 / (spec.c_in // spec.groups * spec.kh * spec.kw))
    w = rng.standard_normal(size=spec.w_shape(), dtype=np.float32) * np.float32(std)
    return quantize(w, spec.dtype)


def gen_bias(spec: ConvSpec, seed: int) -> np.ndarray:
    rng = np.random.default_rng(seed)
    return (rng.standard_normal(size=(spec.c_out,), dtype=np.float32) * np.float32(0.1)).astype(np.float32)


def gen_mask(length: int, keep: int, seed: int) -> np.ndarray:
    """uint8 mask with exactly ``keep`` ones (1 = keep the row, 0 = drop it)."""
    if not 0 <= keep <= length:
        raise ValueError("keep out of range")
    rng = np.random.default_rng(seed)
    mask = np.ones(length, dtype=np.uint8)
    if keep < length:
        drop = rng.permutation(length)[: length - keep]
        mask[drop] = 0
    return mask


def gen_score(h: int, w: int, seed: int) -> np.ndarray:
    """The random 2-D score of the mask generator (Alg. 1), uniform in [0, 1), at the input resolution."""
    return np.random.default_rng(seed).random((h, w), dtype=np.float32)


@dataclass
class ConvInputs:
    spec: ConvSpec
    x: np.ndarray  # float32, values representable in spec.dtype
    w: np.ndarray  # float32, values representable in spec.dtype
    bias: Optional[np.ndarray]  # float32 or None
    mask: np.ndarray  # uint8
    keep: int


def make_conv_inputs(spec: ConvSpec, base_seed: int, x: Optional[np.ndarray] = None) -> ConvInputs:
    """All tensors of one layer.  ``x`` may be supplied (network chains)."""
    li = spec.layer_index
    if x is None:
        x = gen_activations(spec.x_shape(), _seed(base_seed, li, 0), spec.dtype)
    w = gen_weights(spec, _seed(base_seed, li, 1))
    b = gen_bias(spec, _seed(base_seed, li, 2)) if spec.has_bias else None
    keep = n_keep(spec.sparsity, spec.mask_len)
    mask = gen_mask(spec.mask_len, keep, _seed(base_seed, li, 3))
    return ConvInputs(spec=spec, x=x, w=w, bias=b, mask=mask, keep=keep)


# --------------------------------------------------------------------------------------
# the five benchmark configurations
# --------------------------------------------------------------------------------------


def base_seed(config_index: int) -> int:
    return 2309 + int(config_index)


def config1() -> ConvSpec:
    """Single 3x3 conv, fp32, batch 1, 16->16 channels at 16x16, half of the rows dropped."""
    return ConvSpec("c1_conv3x3_16", n=1, c_in=16, h=16, w=16, c_out=16, dtype="f32", sparsity=0.5)


C2_SPARSITIES = (0.0, 0.25, 0.5, 0.7)


def config2(sparsity: float = 0.5) -> ConvSpec:
    """ResNet18 stage-1 conv: batch 32, 64->64 at 56x56, 3x3 stride 1 pad 1, bf16."""
    return ConvSpec("c2_resnet18_layer1", n=32, c_in=64, h=56, w=56, c_out=64, dtype="bf16", sparsity=sparsity)


def config4(batch: int = 64, sparsity: float = 0.5) -> List[ConvSpec]:
    """Pointwise (1x1) MobileNetV2-style layers: 4 channel pairs x 4 resolutions."""
    out = []
    li = 0
    for (ci, co) in ((32, 192), (192, 32), (96, 576), (576, 160)):
        for hw in (56, 28, 14, 7):
            out.append(
                ConvSpec(
                    f"c4_pw_{ci}_{co}_{hw}", n=batch, c_in=ci, h=hw, w=hw, c_out=co, kh=1, kw=1, pad_h=0, pad_w=0,
                    dtype="bf16", sparsity=sparsity, layer_index=li,
                )
            )
            li += 1
    return out


def depthwise_layers(batch: int = 64, sparsity: float = 0.5, dtype: str = "bf16") -> List[ConvSpec]:
    """Depthwise 3x3 layers of a MobileNetV2-style body at 224x224 input (channels, map, stride): the
    second workload the build widens into -- the paper times such networks end to end (Sec. 4) but
    lists no layer shapes, so these are the standard ones of that architecture."""
    shapes = [(32, 112, 1), (96, 112, 2), (144, 56, 1), (144, 56, 2), (192, 28, 1), (192, 28, 2), (384, 14, 1),
              (576, 14, 1), (576, 14, 2), (960, 7, 1)]
    return [ConvSpec(f"dw_{c}_{hw}_s{st}", n=batch, c_in=c, h=hw, w=hw, c_out=c, kh=3, kw=3, stride_h=st, stride_w=st,
                     pad_h=1, pad_w=1, dtype=dtype, relu=True, sparsity=sparsity, layer_index=i, groups=c)
            for i, (c, hw, st) in enumerate(shapes)]


@dataclass(frozen=True)
class NetOp:
    """One node of a small inference graph.

    kind: "conv" (spec set), "maxpool" (3x3 stride 2 pad 1), "add_relu" (out = max(a+b, 0)), "add" (out = a+b).
    Tensors are named; "input" is the synthetic network input; a conv whose ``src``
    starts with "synthetic:" draws its own input from the generator.
    """

    kind: str
    out: str
    src: str
    src2: str = ""
    spec: Optional[ConvSpec] = None


def _resnet18_ops(batch: int, res: int, dtype: str, sparsity: float, sparse_downsample: bool,
                  widths=(64, 128, 256, 512)) -> List[NetOp]:
    ops: List[NetOp] = []
    li = 0

    def conv(name, src, out, ci, co, hw, k, s, p, relu, sp):
        nonlocal li
        spec = ConvSpec(name, n=batch, c_in=ci, h=hw, w=hw, c_out=co, kh=k, kw=k, stride_h=s, stride_w=s,
                        pad_h=p, pad_w=p, dtype=dtype, relu=relu, sparsity=sp, layer_index=li)
        li += 1
        ops.append(NetOp("conv", out, src, spec=spec))
        return spec

    st = conv("stem", "input", "stem", 3, widths[0], res, 7, 2, 3, True, sparsity)
    ops.append(NetOp("maxpool", "pool", "stem"))
    hw = (st.ho + 2 - 3) // 2 + 1
    cur, ch = "pool", widths[0]
    for stage, co in enumerate(widths, start=1):
        for blk in range(2):
            stride = 2 if (stage > 1 and blk == 0) else 1
            tag = f"l{stage}b{blk}"
            c1 = conv(f"{tag}_conv1", cur, f"{tag}_c1", ch, co, hw, 3, stride, 1, True, sparsity)
            conv(f"{tag}_conv2", f"{tag}_c1", f"{tag}_c2", co, co, c1.ho, 3, 1, 1, False, sparsity)
            short = cur
            if stride != 1 or ch != co:
                conv(f"{tag}_down", cur, f"{tag}_ds", ch, co, hw, 1, stride, 0, False,
                     sparsity if sparse_downsample else 0.0)
                short = f"{tag}_ds"
            ops.append(NetOp("add_relu", f"{tag}_out", f"{tag}_c2", short))
            cur, ch, hw = f"{tag}_out", co, c1.ho
    return ops


def config3(batch: int = 64, res: int = 224, sparsity: float = 0.5, sparse_downsample: bool = True,
            dtype: str = "bf16") -> List[NetOp]:
    """ResNet18 convolution stack (20 convs), BN folded into bias, one mask per conv.

    The paper leaves the 1x1 downsample convs dense (App. B.3); ``sparse_downsample=False``
    reproduces that, the default masks every conv as the benchmark description asks.
    """
    return _resnet18_ops(batch, res, dtype, sparsity, sparse_downsample)


def pruned_resnet18(batch: int = 64, res: int = 224, sparsity: float = 0.3, keep: float = 0.8,
                    dtype: str = "bf16") -> List[NetOp]:
    """ResNet18 stack after structured channel pruning: every stage keeps the fraction `keep` of its
    channels (51 / 102 / 205 / 410 at 0.8), counts that are no multiple of 8.  Stands in for the pruned
    models of the paper's Sec. 4.5 and the table of App. B.3 (structured weight pruning combined with activation sparsity at
    5-30 %), whose channel counts the paper does not list."""
    widths = tuple(int(round(c * keep)) for c in (64, 128, 256, 512))
    return _resnet18_ops(batch, res, dtype, sparsity, True, widths)


def pad_channels(ops: List[NetOp], multiple: int = 16) -> List[NetOp]:
    """The same graph with every channel count rounded up to `multiple` (the network input keeps its own):
    how a converter lays out a pruned model for 16-byte channel groups (multiples of 8 channels suffice for
    vectorised gathers and stores; multiples of 16 are what every kernel of the library accepts).  The extra filters and filter
    entries are zero, so the extra channels of every tensor stay zero."""
    up = lambda c: -(-c // multiple) * multiple
    out = []
    for o in ops:
        if o.kind != "conv":
            out.append(o)
            continue
        c_in = o.spec.c_in if o.src == "input" else up(o.spec.c_in)
        out.append(replace(o, spec=o.spec.with_(c_in=c_in, c_out=up(o.spec.c_out))))
    return out


def config5(batch: int = 16, sparsity: float = 0.3, dtype: str = "bf16") -> List[NetOp]:
    """Detector-style backbone at 640x640 (feature maps 80/40/20) plus 1x1 neck convs.

    The backbone is a plain chain; a neck conv whose channel count matches no backbone
    tensor draws its own half-normal input.
    """
    ops: List[NetOp] = []
    li = 0

    def conv(name, src, out, ci, co, hw, k, s):
        nonlocal li
        spec = ConvSpec(name, n=batch, c_in=ci, h=hw, w=hw, c_out=co, kh=k, kw=k, stride_h=s, stride_w=s,
                        pad_h=k // 2, pad_w=k // 2, dtype=dtype, relu=True, sparsity=sparsity, layer_index=li)
        li += 1
        ops.append(NetOp("conv", out, src, spec=spec))

    conv("y1", "input", "y1", 32, 64, 80, 3, 1)
    conv("y2", "y1", "y2", 64, 64, 80, 3, 1)
    conv("y3", "y2", "y3", 64, 128, 80, 3, 2)
    conv("y4", "y3", "y4", 128, 128, 40, 3, 1)
    conv("y5", "y4", "y5", 128, 256, 40, 3, 2)
    conv("y6", "y5", "y6", 256, 256, 20, 3, 1)
    conv("y7", "y6", "y7", 256, 512, 20, 3, 1)
    conv("y8", "y7", "y8", 512, 512, 20, 3, 1)
    conv("neck_512_256_20", "y8", "n1", 512, 256, 20, 1, 1)
    conv("neck_256_128_40", "synthetic:n2", "n2", 256, 128, 40, 1, 1)
    conv("neck_128_64_80", "synthetic:n3", "n3", 128, 64, 80, 1, 1)
    conv("neck_256_256_40", "synthetic:n4", "n4", 256, 256, 40, 1, 1)
    return ops


def mobilenet_v2(batch: int = 64, res: int = 224, sparsity: float = 0.5, dtype: str = "bf16") -> List[NetOp]:
    """Convolution stack of a MobileNetV2-style network (width 1.0): 3x3 stem, one depthwise-separable block,
    sixteen inverted-residual blocks (1x1 expansion by 6 -> depthwise 3x3 -> linear 1x1 projection, identity
    shortcut where shape allows) and the 1x1 head; 52 convs.  BN folded into bias; ReLU stands in for the
    architecture's clipped ReLU (the library has none / ReLU).  The paper times this family end to end
    (Sec. 4) without listing shapes: these are the standard ones.  Every conv is masked with 2-D masks
    (one per layer resolution under Alg. 1's propagation), so all layers of one resolution share a mask."""
    ops: List[NetOp] = []
    li = 0

    def conv(name, src, out, ci, co, hw, k, s, relu, groups=1):
        nonlocal li
        spec = ConvSpec(name, n=batch, c_in=ci, h=hw, w=hw, c_out=co, kh=k, kw=k, stride_h=s, stride_w=s,
                        pad_h=k // 2, pad_w=k // 2, dtype=dtype, relu=relu, sparsity=sparsity, layer_index=li,
                        groups=groups, mask_mode="spatial")
        li += 1
        ops.append(NetOp("conv", out, src, spec=spec))
        return spec

    hw = conv("stem", "input", "stem", 3, 32, res, 3, 2, True).ho
    conv("b0_dw", "stem", "b0_d", 32, 32, hw, 3, 1, True, groups=32)
    conv("b0_project", "b0_d", "b0_out", 32, 16, hw, 1, 1, False)
    cur, ch, blk = "b0_out", 16, 1
    for expand, co, repeats, stride in [(6, 24, 2, 2), (6, 32, 3, 2), (6, 64, 4, 2), (6, 96, 3, 1), (6, 160, 3, 2),
                                        (6, 320, 1, 1)]:
        for r in range(repeats):
            st = stride if r == 0 else 1
            mid, tag = ch * expand, f"b{blk}"
            conv(f"{tag}_expand", cur, f"{tag}_e", ch, mid, hw, 1, 1, True)
            d = conv(f"{tag}_dw", f"{tag}_e", f"{tag}_d", mid, mid, hw, 3, st, True, groups=mid)
            conv(f"{tag}_project", f"{tag}_d", f"{tag}_p", mid, co, d.ho, 1, 1, False)
            out = f"{tag}_p"
            if st == 1 and ch == co:
                ops.append(NetOp("add", f"{tag}_out", f"{tag}_p", cur))
                out = f"{tag}_out"
            cur, ch, hw, blk = out, co, d.ho, blk + 1
    conv("head", cur, "head", ch, 1280, hw, 1, 1, True)
    return ops


def with_spatial_masks(ops: List[NetOp]) -> List[NetOp]:
    """The same graph with one 2-D mask per conv layer shared by the batch (the paper's mask shape)."""
    return [replace(o, spec=o.spec.with_(mask_mode="spatial")) if o.kind == "conv" else o for o in ops]


def network_input_shape(ops: List[NetOp]):
    first = next(o for o in ops if o.kind == "conv" and o.src == "input")
    return first.spec.x_shape()


def conv_specs(ops: List[NetOp]) -> List[ConvSpec]:
    return [o.spec for o in ops if o.kind == "conv"]


def conv_flops(spec: ConvSpec, keep: Optional[int] = None) -> float:
    """Algorithmic FLOPs of the contraction on ``keep`` rows (all rows if None)."""
    rows = spec.m if keep is None else keep
    return 2.0 * rows * spec.k * spec.c_out
