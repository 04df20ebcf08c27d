"""Inverted-residual stack (1x1 expansion -> depthwise 3x3 -> linear 1x1 projection, shortcuts) with masks
from the GPU generator: every tensor against the CPU oracle, once with dense tensors throughout and once
with the narrow tensors kept as compact [kept x C] matrices between the layers that share a mask."""
import numpy as np
import pytest
import torch

import paper_2309_06626_amd.binding as B
import paper_2309_06626_amd.runtime as R
import workloads as W
from oracle import mask_oracle as MO
from oracle import oracle
from parity import TOL

pytestmark = pytest.mark.gpu


def build(dtype, batch, res, sparsity, seed):
    ops = W.mobilenet_v2(batch=batch, res=res, sparsity=sparsity, dtype=dtype)
    score = W.gen_score(res, res, seed=seed + 5)
    score_dev = torch.from_numpy(score).to("cuda:0")
    params, layers = {}, {}
    for spec in W.conv_specs(ops):
        ci = W.make_conv_inputs(spec, seed, x=np.zeros(1, np.float32))
        want = MO.layer_mask(score, spec.ho, spec.wo, float(np.float32(spec.sparsity))).reshape(-1)
        got = B.sparse_mask_generate(score_dev, spec.ho, spec.wo, spec.sparsity)
        torch.cuda.synchronize()
        assert np.array_equal(got.cpu().numpy().reshape(-1), want), spec.name
        params[spec.name] = (ci.w, ci.bias, want)
        layers[spec.name] = R.ConvLayer(spec, ci.w, ci.bias, want)
    host = {"input": W.gen_activations(W.network_input_shape(ops), seed, dtype)}
    return ops, params, layers, host


def dense_view(op_out, t, ops, layers, fmt):
    """Host float32 [N, Ho, Wo, C] view of a device tensor, compact tensors scattered back by the row list."""
    if not fmt.get(op_out, False):
        return R.to_host_f32(t)
    # the row list of a compact tensor is that of the conv that made it (or of the operands of a sum)
    op = next(o for o in ops if o.out == op_out)
    while op.kind != "conv":
        op = next(o for o in ops if o.out == op.src)
    spec = op.spec
    rows = B.plan_row_idx(layers[spec.name].plan).cpu().numpy()
    c = t.shape[1]
    out = np.zeros((spec.m, c), np.float32)
    out[rows] = R.to_host_f32(t)
    return out.reshape(spec.n, spec.ho, spec.wo, c)


def compare(ops, dev, ref, params, layers, fmt, tol, what):
    for op in ops:
        g, r = dense_view(op.out, dev[op.out], ops, layers, fmt), ref[op.out]
        assert g.shape == r.shape, f"{what} {op.out}"
        assert np.isfinite(g).all(), f"{what} {op.out}"
        nr = np.linalg.norm(r.astype(np.float64))
        err = np.linalg.norm(g.astype(np.float64) - r) / max(nr, 1e-30)
        assert err <= tol, f"{what} {op.out}: normwise {err:.3e}"
        assert np.abs(g - r).max() <= tol * max(np.abs(r).max(), 1e-30), f"{what} {op.out}"
        if op.kind == "conv" and not fmt.get(op.out, False):
            s = op.spec
            mask = np.tile(params[s.name][2], s.n)
            bits = R.bits_of(dev[op.out]).reshape(s.m, s.c_out)
            assert (bits[mask == 0] == 0).all(), f"{what} {op.out}: dropped rows must be zero"


@pytest.mark.parametrize("dtype,batch,res,sparsity,dw_compact", [("bf16", 2, 96, 0.5, True), ("f16", 1, 64, 0.3, False),
                                                                  ("f16", 2, 64, 0.5, True)])
def test_inverted_residual_stack_dense_and_compact_formats(dtype, batch, res, sparsity, dw_compact, monkeypatch):
    if dw_compact:    # (the maps are small here: lift the size rule so that the depthwise layers read compact inputs too)
        monkeypatch.setattr(R, "kCompactDepthwiseInput", 0)
    ops, params, layers, host = build(dtype, batch, res, sparsity, seed=900)
    ref = oracle.run_network(ops, host, lambda spec: params[spec.name])
    tol = TOL[dtype]
    x = {k: R.to_device(v, dtype) for k, v in host.items()}
    # dense tensors everywhere
    dev = R.run_network(ops, x, layers)
    torch.cuda.synchronize()
    compare(ops, dev, ref, params, layers, {}, tol, "dense tensors")
    # compact tensors wherever the graph allows
    fmt = R.plan_row_formats(ops, layers)
    assert sum(fmt.values()) == (len(ops) - 1 if dw_compact else 44)
    assert fmt["b2_out"] and fmt["b5_d"] and fmt["b5_e"] == dw_compact and not fmt["head"]
    runner = R.NetworkRunner(ops, x, layers, row_formats=fmt)
    for name, t in runner.tensors.items():
        if name != "input":
            t.fill_(float("nan"))
    out = runner.run()
    torch.cuda.synchronize()
    assert out["b2_out"].dim() == 2 and out["b2_out"].shape[0] == layers["b2_project"].info["kept"]
    compare(ops, out, ref, params, layers, fmt, tol, "compact tensors")
    # both formats hold the same numbers: every kernel computes a kept row the same way
    for op in ops:
        a = dense_view(op.out, dev[op.out], ops, layers, {})
        b = dense_view(op.out, out[op.out], ops, layers, fmt)
        assert np.allclose(a, b, rtol=4 * tol, atol=4 * tol * max(np.abs(a).max(), 1e-30)), op.out
    # replayed as a HIP graph, several times with eager work in between
    first = {k: v.clone() for k, v in out.items()}
    graph = runner.capture()
    for _ in range(3):
        for name, t in runner.tensors.items():
            if name != "input":
                t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k, v in runner.tensors.items():
            assert torch.equal(v.view(torch.int16), first[k].view(torch.int16)), k
