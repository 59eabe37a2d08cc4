"""Whole-model pins: structural facts of the five architectures, the graph
plumbing of the oracle's model runner (against a library forward pass in fp64
built from the same description), and the cross-mode / cross-precision bounds.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from workloads import gen, randnet, zoo

import json
import os

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
ARCH = {k: v for k, v in json.load(open(os.path.join(GOLDEN, "architectures.json"))).items() if not k.startswith("_")}


@pytest.mark.parametrize("fam", sorted(ARCH))
def test_structure(fam):
    """Node, parameter and MAC counts of the published architecture tables (tests/golden/architectures.json)."""
    g = ARCH[fam]
    m = zoo.FAMILIES[fam]()
    ops = [L.op for L in m.layers]
    assert len(ops) == g["nodes"]
    assert (ops.count("conv"), ops.count("dwconv"), ops.count("maxpool"), ops.count("gap"), ops.count("fc")) == \
        (g["conv"], g["dwconv"], g["maxpool"], g["gap"], g["fc"])
    assert ops.count("concat") == g.get("concat", 0) and ops.count("avgpool") == g.get("avgpool", 0) and ops.count("mul") == g.get("mul", 0)
    assert ops.count("slice") == g.get("slice", 0) and ops.count("shuffle") == g.get("shuffle", 0)
    assert max(m.levels()) == g["depth"]
    assert m.n_params() == g["params"]
    assert m.macs() == g["macs"]
    assert m.layers[m.output].cout == g["classes"]
    if "gmacs_published" in g:
        affine = sum(L.out_h * L.out_w * L.cout for L in m.layers if L.op == "dwconv" and L.k == 1 and not L.bn)
        assert affine == g.get("affine_macs", 0)
        assert round((m.macs() - affine) / 1e9, 2) == g["gmacs_published"]
    if "params_with_batchnorm" in g:  # folding removes one of BatchNorm's two parameters per normalised channel
        bn_channels = sum(L.cout for L in m.layers if L.op in ("conv", "dwconv") and L.bn and L.bias)
        assert g["params_with_batchnorm"] - g["params"] in (bn_channels, 0)


def test_config1_matches_stored_oracle_values():
    """The oracle reproduces its stored outputs for configuration 1 (a guard against silent oracle drift)."""
    gold = json.load(open(os.path.join(GOLDEN, "config1_oracle.json")))
    x = gen.make_input(7, 1, 3, 32, 32, "uniform", "f32")
    for i, mem in enumerate(gold["members"]):
        m = zoo.tiny_cnn("f32", softmax=True)
        blob = gen.make_blob(m, mem["seed"], bias_std=0.0)
        logits = oracle.run_model(m, blob, x, node=4)[0]
        probs = oracle.run_model(m, blob, x)[0]
        assert np.allclose(logits, mem["logits"], rtol=1e-6, atol=1e-7)
        assert np.allclose(probs, mem["softmax"], rtol=1e-6, atol=1e-8)
        assert int(oracle.top1(logits[None])[0]) == mem["top1"]


def test_stage_shapes():
    r = zoo.resnet50()
    sides = [L.out_h for L in r.layers if L.op == "conv"]
    assert sides[0] == 112 and set(sides) == {112, 56, 28, 14, 7}
    assert r.layers[1].op == "maxpool" and r.layers[1].out_h == 56
    v = zoo.vgg16()
    assert [L.out_h for L in v.layers if L.op == "maxpool"] == [112, 56, 28, 14, 7]
    assert [L.cin for L in v.layers if L.op == "fc"] == [25088, 4096, 4096]
    mb = zoo.mobilenetv2()
    dw = [L for L in mb.layers if L.op == "dwconv"]
    assert [L.cout for L in dw][:4] == [32, 96, 144, 144] and dw[-1].cout == 960 and dw[-1].out_h == 7
    assert sum(1 for L in mb.layers if L.residual >= 0) == 10
    assert sum(1 for L in zoo.resnet50().layers if L.residual >= 0) == 16


def _torch_forward(model, blob, x, dtype=torch.float64):
    """Library forward pass in fp64 from the same description (no oracle code)."""
    vals = []
    xt = torch.from_numpy(x).to(dtype)
    for L in model.layers:
        inp = xt if L.input == -1 else vals[L.input]
        if L.op in ("conv", "dwconv", "fc"):
            nw = {"conv": L.cout * (L.cin // L.groups) * L.k * (L.kw or L.k), "dwconv": L.cout * L.k * L.k, "fc": L.cout * L.cin}[L.op]
            if model.dtype == "f32":
                w = blob[L.w_off:L.w_off + 4 * nw].view(np.float32)
            else:
                w = gen.bf16_to_f32(blob[L.w_off:L.w_off + 2 * nw].view(np.uint16))
            w = torch.from_numpy(np.array(w)).to(dtype)
            b = torch.from_numpy(np.array(blob[L.b_off:L.b_off + 4 * L.cout].view(np.float32))).to(dtype)
        if L.op == "conv":
            kw = L.kw or L.k
            pad = (L.pad, L.pad) if kw == L.k else (L.pad if L.k > 1 else 0, L.pad if kw > 1 else 0)
            y = F.conv2d(inp, w.reshape(L.cout, L.cin // L.groups, L.k, kw), b, stride=L.stride, padding=pad, groups=L.groups)
        elif L.op == "dwconv":
            y = F.conv2d(inp, w.reshape(L.cout, 1, L.k, L.k), b, stride=L.stride, padding=L.pad, groups=L.cout)
        elif L.op == "maxpool":
            y = F.max_pool2d(inp, L.k, L.stride, L.pad, ceil_mode=bool(L.ceil))
        elif L.op == "mul":
            y = inp * vals[L.residual]
        elif L.op == "slice":
            y = inp[:, L.first:L.first + L.cout]
        elif L.op == "shuffle":
            n_, c_, h_, w_ = inp.shape
            y = inp.view(n_, L.groups, c_ // L.groups, h_, w_).transpose(1, 2).reshape(n_, c_, h_, w_)
        elif L.op == "avgpool":
            y = F.avg_pool2d(inp, L.k, L.stride, L.pad)
        elif L.op == "concat":
            y = torch.cat([inp, vals[L.residual]], dim=1)
        elif L.op == "gap":
            y = inp.mean(dim=(2, 3), keepdim=True)
        elif L.op == "fc":
            y = F.linear(inp.reshape(inp.shape[0], -1), w.reshape(L.cout, L.cin), b).reshape(-1, L.cout, 1, 1)
        elif L.op == "softmax":
            y = torch.softmax(inp.reshape(inp.shape[0], -1), dim=1).reshape(inp.shape)
        if L.residual >= 0 and L.op not in ("concat", "mul"):
            y = y + vals[L.residual]
        if L.act == "relu":
            y = torch.relu(y)
        elif L.act == "relu6":
            y = torch.clamp(y, 0.0, 6.0)
        elif L.act != "none":
            y = {"hardswish": F.hardswish, "hardsigmoid": F.hardsigmoid, "silu": F.silu, "sigmoid": torch.sigmoid}[L.act](y)
        vals.append(y)
    return vals[-1].reshape(x.shape[0], -1).numpy()


def _rel(a, b):
    return float(np.linalg.norm(a.astype(np.float64) - b) / np.linalg.norm(b))


@pytest.mark.parametrize("fam,hw", [("tiny", 32), ("resnet18", 64), ("resnet50", 64), ("mobilenetv2", 64), ("vgg16", 32),
                                    ("alexnet", 67), ("mnasnet1_0", 64), ("squeezenet1_1", 65), ("googlenet", 70), ("resnext50_32x4d", 64), ("densenet121", 64), ("mobilenet_v3_large", 64), ("mobilenet_v3_small", 64), ("shufflenet_v2_x1_0", 64), ("inception_v3", 96)])
def test_model_runner_vs_library_forward(fam, hw):
    m = zoo.tiny_cnn() if fam == "tiny" else zoo.FAMILIES[fam](hw=hw)
    blob = gen.make_blob(m, 1000 + hw)
    x = gen.make_input(7, 2, 3, hw, hw, "uniform" if fam == "tiny" else "normal", m.dtype)
    ref = _torch_forward(m, blob, x)
    y = oracle.run_model(m, blob, x, round_storage=False)
    assert y.shape == ref.shape
    assert _rel(y, ref) < 2e-5
    # the double-accumulation build bounds the oracle's own rounding
    y64 = oracle.run_model(m, blob, x, round_storage=False, f64=True)
    assert _rel(y64, ref) < 2e-6
    assert _rel(y, y64.astype(np.float64)) < 1e-5
    # batch independence: image 1 alone gives image 1's row, bit for bit
    y1 = oracle.run_model(m, blob, x[1:2], round_storage=False)
    assert np.array_equal(y1[0], y[1])


@pytest.mark.parametrize("seed", range(40))
def test_random_graphs_vs_library_forward(seed):
    """Random layer graphs over every operator (odd channel counts, non-square inputs, residuals and
    concatenations across distant nodes): the oracle's model runner against the library forward pass."""
    m = randnet.random_model(seed, max_nodes=12)
    blob = gen.make_blob(m, 5000 + seed)
    x = gen.make_input(11 + seed, 2, m.in_c, m.in_h, m.in_w, "normal", m.dtype)
    ref = _torch_forward(m, blob, x)
    y = oracle.run_model(m, blob, x, round_storage=False)
    assert y.shape == ref.shape and np.isfinite(y).all()
    scale = np.linalg.norm(ref)
    assert np.linalg.norm(y.astype(np.float64) - ref) <= 2e-5 * scale + 1e-6
    y64 = oracle.run_model(m, blob, x, round_storage=False, f64=True)
    assert np.linalg.norm(y64 - ref) <= 2e-6 * scale + 1e-9


def test_residual_is_added_before_activation():
    m = zoo.Model("r", "f32", 2, 3, 3)
    a = m.add(zoo.CONV, -1, cin=2, cout=2, k=1, stride=1, pad=0, act=zoo.NONE)
    m.add(zoo.CONV, a, cin=2, cout=2, k=1, stride=1, pad=0, act=zoo.RELU, residual=a)
    m.shapes()
    size = gen.layout_blob(m)
    blob = np.zeros(size, np.uint8)
    eye = np.eye(2, dtype=np.float32).reshape(-1)
    for L in m.layers:
        blob[L.w_off:L.w_off + 16] = eye.view(np.uint8)
    x = np.array([-3.0, 2.0] * 9, dtype=np.float32).reshape(1, 3, 3, 2).transpose(0, 3, 1, 2).copy()
    y = oracle.run_model(m, blob, x).reshape(1, 2, 3, 3)
    assert np.all(y[0, 0] == 0.0)  # relu(-3 + -3) = 0, not -3 + relu(-3)
    assert np.all(y[0, 1] == 4.0)


def test_storage_rounding_mode_scale():
    """Mode S differs from mode F by roughly sqrt(#roundings) * 2^-9 and every stored value is bf16."""
    m = zoo.resnet18(hw=64)
    blob = gen.make_blob(m, 1000)
    x = gen.make_input(7, 1, 3, 64, 64, "normal", "bf16")
    yf = oracle.run_model(m, blob, x, round_storage=False)
    ys = oracle.run_model(m, blob, x, round_storage=True)
    d = _rel(ys, yf.astype(np.float64))
    assert 1e-4 < d < 1e-2
    mid = oracle.run_model(m, blob, x, round_storage=True, node=5)
    assert np.array_equal(mid, oracle.round_bf16(mid))  # an interior node is stored as bf16
    assert not np.array_equal(ys, oracle.round_bf16(ys))  # logits stay fp32


def test_softmax_output_keeps_fp32_logits():
    m = zoo.tiny_cnn("bf16")
    blob = gen.make_blob(m, 5, bias_std=0.0)
    x = gen.make_input(7, 1, 3, 32, 32, "uniform", "bf16")
    logits = oracle.run_model(m, blob, x, round_storage=True, node=4)
    p = oracle.run_model(m, blob, x, round_storage=True)
    assert np.allclose(p, oracle.softmax(logits), atol=1e-7)
    assert abs(p.sum() - 1.0) < 1e-6
