"""Host logic that decides which tensors of a network stay compact (no GPU needed)."""
from types import SimpleNamespace

import workloads as W
from paper_2309_06626_amd import runtime as R


def stub_layers(ops, key_of):
    return {s.name: SimpleNamespace(rows_key=key_of(s)) for s in W.conv_specs(ops)}


def by_resolution(spec):
    """Propagated masks: one row list per output resolution."""
    return (spec.n, spec.ho, spec.wo)


def test_inverted_residual_blocks_keep_their_narrow_tensors_compact(monkeypatch):
    ops = W.mobilenet_v2(batch=2, res=96)
    fmt = R.plan_row_formats(ops, stub_layers(ops, by_resolution))
    for op in ops:
        name = op.out
        if op.kind == "add":
            assert fmt[name], name                       # shortcuts add compact matrices
        elif name == "stem" or name.endswith("_e") or name == "head":
            assert not fmt[name], name                   # small maps: depthwise layers read dense inputs; graph output
        else:
            assert fmt[name], name                       # depthwise and projection outputs feed 1x1 layers
    assert sum(fmt.values()) == 17 + 17 + 10             # 17 depthwise, 17 projections, 10 shortcuts
    # large maps: the depthwise layers read compact inputs as well
    monkeypatch.setattr(R, "kCompactDepthwiseInput", 0)
    fmt = R.plan_row_formats(ops, stub_layers(ops, by_resolution))
    assert all(fmt[op.out] == (op.out != "head") for op in ops)
    # at full size the threshold separates the first blocks from the rest
    monkeypatch.undo()
    ops = W.mobilenet_v2(batch=64, res=224)
    fmt = R.plan_row_formats(ops, stub_layers(ops, by_resolution))
    assert fmt["stem"] and fmt["b1_e"] and fmt["b2_e"] and fmt["b3_e"] and not fmt["b4_e"] and not fmt["b16_e"]


def test_different_masks_or_window_layers_force_dense_tensors(monkeypatch):
    monkeypatch.setattr(R, "kCompactDepthwiseInput", 0)
    ops = W.mobilenet_v2(batch=2, res=96)
    # every layer with a mask of its own: only the depthwise layers (which look pixels up in their input's row
    # list, whatever their own mask) can take a compact map
    fmt = R.plan_row_formats(ops, stub_layers(ops, lambda s: s.name))
    assert all(fmt[n] == (n == "stem" or n.endswith("_e")) for n in fmt), fmt
    # ResNet18: every tensor feeds a 3x3 layer, a strided 1x1 layer or the output
    ops = W.with_spatial_masks(W.config3(batch=1, res=64))
    fmt = R.plan_row_formats(ops, stub_layers(ops, by_resolution))
    assert not any(fmt.values())


def test_dense_shortcut_operand_makes_the_whole_sum_dense(monkeypatch):
    monkeypatch.setattr(R, "kCompactDepthwiseInput", 0)
    ops = W.mobilenet_v2(batch=1, res=64)
    layers = stub_layers(ops, by_resolution)
    layers["b1_project"].rows_key = "other"             # b1_p is read by b2_expand and by the shortcut of block 2
    fmt = R.plan_row_formats(ops, layers)
    assert not fmt["b1_p"] and not fmt["b2_out"] and not fmt["b2_p"]
    assert fmt["b2_d"] and fmt["b2_e"] and fmt["b4_out"]
