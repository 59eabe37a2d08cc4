"""Whole-configuration GPU parity: the five benchmark configurations through the
C-ABI, against the CPU oracle on the same seeded inputs, at full size and in the
launch configuration the benchmark times (grouped levels, one-copy load).

Tolerances: relative L2 <= 1e-2 on logits for bf16 members against the
fp32-activation oracle (mode F), <= 1e-4 for fp32; top-1 identical, judged against the
oracle run with the same storage rounding (mode S), a near tie being reported, never dropped.
MobileNetV2 with these synthetic weights amplifies bf16 storage noise about tenfold (the
oracle's own mode S sits 2e-2 from mode F), so that member keeps fp32 activations.
"""
import numpy as np
import pytest

from workloads import gen, zoo

pytestmark = pytest.mark.gpu

WIDE = {"mobilenetv2"}  # members whose activations stay fp32


def _member(fam, seed, **kw):
    m = zoo.FAMILIES[fam](**kw)
    return (m, gen.make_blob(m, seed), "f32" if fam in WIDE else None)


def _check_member(name, y, ref_f, ref_s, tol):
    from tests import harness
    harness.check_member(name, y, ref_f, ref_s, wide=tol < 1e-3, tol=tol)


def test_config1_two_tiny_cnns_fp32():
    from tests import harness
    import oracle
    x = gen.make_input(7, 1, 3, 32, 32, "uniform", "f32")
    for softmax in (True, False):
        mem = []
        for i in range(2):
            m = zoo.tiny_cnn("f32", softmax=softmax)
            mem.append((m, gen.make_blob(m, 1000 + i, bias_std=0.0)))
        g = harness.GpuDag(mem, 1)
        try:
            ys = g.run(x)
        finally:
            g.close()
        import json
        import os
        gold = json.load(open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "config1_oracle.json")))
        for i, ((m, blob), y) in enumerate(zip(mem, ys)):
            ref = oracle.run_model(m, blob, x)
            assert harness.rel_l2(y, ref) <= 1e-4
            stored = np.array(gold["members"][i]["softmax" if softmax else "logits"], dtype=np.float32)[None]
            assert harness.rel_l2(y, stored) <= 1e-4  # the oracle's stored values (tests/golden)
            assert int(oracle.top1(y)[0]) == int(oracle.top1(ref)[0])
            if softmax:
                assert abs(float(y.sum()) - 1.0) < 1e-5
        assert not np.array_equal(ys[0], ys[1])


def test_config2_two_resnet18_batch1():
    from tests import harness
    mem = [_member("resnet18", 1000 + i) for i in range(2)]
    x = gen.make_input(7, 1, 3, 224, 224, "normal", "bf16")
    g = harness.GpuDag(mem, 1)
    try:
        ys = g.run(x)
    finally:
        g.close()
    refs = harness.oracle_units([(m, b, x, rs) for (m, b, _) in mem for rs in (False, True)])
    for i, (m, b, _) in enumerate(mem):
        _check_member(f"resnet18[{i}]", ys[i], refs[2 * i], refs[2 * i + 1], 1e-2)


def test_config3_heterogeneous_batch8():
    from tests import harness
    fams = ["resnet50", "mobilenetv2", "vgg16"]
    mem = [_member(f, 1000 + i) for i, f in enumerate(fams)]
    x = gen.make_input(7, 8, 3, 224, 224, "normal", "bf16")
    g = harness.GpuDag(mem, 8)
    try:
        ys = g.run(x)
    finally:
        g.close()
    units = []
    for (m, b, act) in mem:
        for img in range(8):
            units.append((m, b, x[img:img + 1], False))
            units.append((m, b, x[img:img + 1], act is None))
    res = harness.oracle_units(units)
    for i, f in enumerate(fams):
        ref_f = np.concatenate([res[(i * 8 + img) * 2] for img in range(8)])
        ref_s = np.concatenate([res[(i * 8 + img) * 2 + 1] for img in range(8)])
        _check_member(f, ys[i], ref_f, ref_s, 1e-4 if f in WIDE else 1e-2)


def test_config4_eight_resnet50_batch32_every_row():
    """Full size on the GPU, in the launch configuration the benchmark times.  Every one of the 32 image rows of
    every one of the 8 members is compared with the oracle, in its fp32-activation mode (relative L2) and in its
    storage-rounding mode (element-wise bound, top-1): Section III-A, C1 holds for every image, the ragged last
    tile of the last stage (image 31) included."""
    from tests import harness
    mem = [_member("resnet50", 1000 + i) for i in range(8)]
    x = gen.make_input(7, 32, 3, 224, 224, "normal", "bf16")
    g = harness.GpuDag(mem, 32)
    try:
        ys = g.run(x)
    finally:
        g.close()
    units = []
    for (m, b, _) in mem:
        for img in range(32):
            units.append((m, b, x[img:img + 1], False))
            units.append((m, b, x[img:img + 1], True))
    res = harness.oracle_units(units)
    for i in range(8):
        ref_f = np.concatenate([res[(i * 32 + j) * 2] for j in range(32)])
        ref_s = np.concatenate([res[(i * 32 + j) * 2 + 1] for j in range(32)])
        _check_member(f"resnet50[{i}]", ys[i], ref_f, ref_s, 1e-2)
    assert not np.array_equal(ys[0], ys[1])


@pytest.mark.parametrize("fam", ["resnext50_32x4d", "densenet121", "googlenet", "squeezenet1_1"])
def test_full_size_family_batch32_sampled(fam):
    """Two identical-architecture members at the family's full image size and batch 32, the launch configuration the
    per-family benchmark times (64-column group-walking tiles for ResNeXt; dense blocks written in place with the
    affine stage applied by the 1x1 convolutions for DenseNet; Inception modules and fire modules written in place,
    four-output pooling strips); the oracle checks four images per member, the first and the last of the batch
    among them (the last owns the ragged tail tile of every layer)."""
    from tests import harness
    mem = [_member(fam, 2000 + i) for i in range(2)]
    hw = mem[0][0].in_h
    x = gen.make_input(9, 32, 3, hw, hw, "normal", "bf16")
    g = harness.GpuDag(mem, 32)
    try:
        ys = g.run(x)
    finally:
        g.close()
    units, picks = [], []
    for i, (m, b, _) in enumerate(mem):
        imgs = [0, (3 + 11 * i) % 32, (30 - 7 * i) % 32, 31]
        picks.append(imgs)
        for img in imgs:
            units.append((m, b, x[img:img + 1], False))
            units.append((m, b, x[img:img + 1], True))
    res = harness.oracle_units(units)
    for i in range(2):
        ref_f = np.concatenate([res[(i * 4 + j) * 2] for j in range(4)])
        ref_s = np.concatenate([res[(i * 4 + j) * 2 + 1] for j in range(4)])
        _check_member(f"{fam}[{i}]", ys[i][picks[i]], ref_f, ref_s, 1e-2)
        assert np.isfinite(ys[i]).all()
    assert not np.array_equal(ys[0], ys[1])


def test_further_table3_families_fused():
    """Further families of the paper's Table III (AlexNet, VGG-11/13/19, ResNet-34/101/152, Wide ResNet-50-2/101-2,
    MnasNet 1.0; SqueezeNet 1.0 / 1.1 and GoogLeNet with channel concatenation and pooling sizes that round up; ResNeXt-50
    32x4d with grouped convolution; DenseNet-121 with window average pooling and per-channel affine nodes; MobileNetV3 Large with squeeze-excite gates
    and hard-swish; ShuffleNet V2 with channel slices and shuffles; Inception v3 with rectangular kernels), all eighteen fused in one DAG at a reduced image size, each member against the oracle.  MnasNet is a MobileNet-style inverted-residual network and keeps fp32 activations."""
    from tests import harness
    WIDE_HERE = {"mnasnet1_0", "mobilenet_v3_large"}   # inverted-residual networks keep fp32 activations
    fams = ["alexnet", "vgg11", "vgg13", "vgg19", "resnet34", "resnet101", "resnet152", "wide_resnet50_2", "wide_resnet101_2", "mnasnet1_0",
            "squeezenet1_0", "squeezenet1_1", "googlenet", "resnext50_32x4d", "densenet121", "mobilenet_v3_large", "shufflenet_v2_x1_0", "inception_v3"]
    mem = []
    for i, f in enumerate(fams):
        m = zoo.FAMILIES[f](hw=96)
        mem.append((m, gen.make_blob(m, 1000 + i), "f32" if f in WIDE_HERE else None))
    x = gen.make_input(7, 2, 3, 96, 96, "normal", "bf16")
    g = harness.GpuDag(mem, 2)
    try:
        ys = g.run(x)
    finally:
        g.close()
    units = []
    for (m, b, act) in mem:
        units.append((m, b, x, False))
        units.append((m, b, x, act is None))
    res = harness.oracle_units(units)
    for i, f in enumerate(fams):
        tol = 1e-2
        if f in WIDE_HERE:
            # fp32-stored activations enter the matrix cores as two bf16 terms, hi = bf16(x) and lo = bf16(x - hi): 16
            # mantissa bits where bf16 storage keeps 8.  Per layer that is 2^-8 of the perturbation bf16 storage makes
            # (pinned on the CPU in tests/test_oracle_pins.py), and both travel through the same graph, so the member
            # ends 2^-8 x (distance between the oracle's storage-rounding and fp32 modes) from the fp32 oracle.  The bar
            # is twice that (summation order adds its own share), and never below the 1e-4 of the fp32 path.
            import oracle
            m, b, _ = mem[i]
            d_sf = harness.rel_l2(oracle.run_model(m, b, x, round_storage=True), res[2 * i])
            tol = max(1e-4, 2.0 * 2.0 ** -8 * d_sf)
            print(f"  {f}: oracle modes S and F differ by {d_sf:.3e}: bar {tol:.3e}")
        _check_member(f, ys[i], res[2 * i], res[2 * i + 1], tol)


def test_remaining_table3_families_fused():
    """The family members of Table III not covered above (DenseNet-169 / 201 / 161 with its 48-channel growth, ResNeXt-101
    32x8d, MobileNetV3-Small, ShuffleNet V2 x0.5), fused in one DAG at a reduced image size, bf16 storage, each against
    the oracle."""
    from tests import harness
    fams = ["densenet169", "densenet201", "densenet161", "resnext101_32x8d", "mobilenet_v3_small", "shufflenet_v2_x0_5"]
    mem = []
    for i, f in enumerate(fams):
        m = zoo.FAMILIES[f](hw=64)
        mem.append((m, gen.make_blob(m, 1100 + i), None))
    x = gen.make_input(17, 2, 3, 64, 64, "normal", "bf16")
    g = harness.GpuDag(mem, 2)
    try:
        ys = g.run(x)
    finally:
        g.close()
    units = []
    for (m, b, act) in mem:
        units.append((m, b, x, False))
        units.append((m, b, x, True))
    res = harness.oracle_units(units)
    for i, f in enumerate(fams):
        _check_member(f, ys[i], res[2 * i], res[2 * i + 1], 1e-2)


def test_efficientnet_v2_prefix():
    """EfficientNetV2-S with these synthetic weights is ill-conditioned as a whole: its activations grow by orders
    of magnitude through 40 residual blocks and the oracle's own fp32 and fp64-accumulation builds end 0.7 apart in
    relative L2, so the full model has no meaningful parity target (parity unpinned).  The prefix through the second
    squeeze-excite block (fused blocks, depthwise blocks, SiLU, sigmoid gate), where the two oracle builds still
    agree to 1e-5, is held to the fp32-activation bar."""
    import copy
    import oracle
    from tests import harness
    full = zoo.FAMILIES["efficientnet_v2_s"](hw=96)
    cut = [i for i, L in enumerate(full.layers) if L.op == "mul"][1] + 1     # the projection after the second gate
    m = zoo.Model("efficientnet_v2_s_prefix", "bf16", 3, 96, 96)
    m.layers = [copy.copy(L) for L in full.layers[:cut + 1]]
    m.shapes()
    blob = gen.make_blob(m, 1016)
    x = gen.make_input(7, 2, 3, 96, 96, "normal", "bf16")
    y32 = oracle.run_model(m, blob, x, round_storage=False)
    y64 = oracle.run_model(m, blob, x, round_storage=False, f64=True)
    assert harness.rel_l2(y32, y64) < 1e-5                                    # the target itself is well conditioned here
    g = harness.GpuDag([(m, blob, "f32")], 2)
    try:
        y = g.run(x)[0]
    finally:
        g.close()
    e = harness.rel_l2(y, harness.oracle_nhwc(m, blob, x, False))
    print(f"  efficientnet_v2_s prefix ({cut + 1} nodes): relL2 {e:.3e}")
    assert e <= 1e-4


def test_config5_swap_churn_all_requests():
    """Pool of 16 packed models, seeded Poisson request stream; per request build, load, run, unload.
    By the fused == alone invariant a member's correct output depends only on (model, input batch), so
    the oracle's logits are memoised per (model, batch) -- all 8 images, both oracle modes -- and every one of
    the 1000 requests is replayed and every row of every member checked by lookup."""
    from tests import harness
    import paper_2410_21120_amd as fi
    import torch
    fams = ["resnet18", "resnet50", "mobilenetv2", "vgg16"]
    pool = []
    for i in range(16):
        fam = fams[i // 4]
        m = zoo.FAMILIES[fam]()
        blob = gen.make_blob(m, 1000 + i)
        act = "f32" if fam in WIDE else None
        spec, keep = fi.make_spec(m, blob.ctypes.data, blob.nbytes, act_dtype=act)
        n = fi.fi_model_packed_size(spec)
        packed = torch.empty(n, dtype=torch.uint8, pin_memory=True)
        fi.fi_model_pack(spec, packed.data_ptr(), n)
        pool.append((m, blob, act, packed))
    batches = [gen.make_input(7 + j, 8, 3, 224, 224, "normal", "bf16") for j in range(2)]
    sample = list(range(8))
    reqs = gen.request_stream(2024, 1000, 16, 4, 50.0, 2)
    assert len(reqs) == 1000
    used = sorted({(mi, bi) for _, mm, bi in reqs for mi in mm})
    units = []
    for mi, bi in used:
        m, blob, act, _ = pool[mi]
        for img in sample:
            units.append((m, blob, batches[bi][img:img + 1], False))
            units.append((m, blob, batches[bi][img:img + 1], act is None))
    res = harness.oracle_units(units)
    memo = {}
    for k, (mi, bi) in enumerate(used):
        base = k * len(sample) * 2
        memo[(mi, bi)] = (np.concatenate([res[base + 2 * j] for j in range(len(sample))]),
                          np.concatenate([res[base + 2 * j + 1] for j in range(len(sample))]))
    alloc = fi.TorchAllocators("cuda:0")
    stream = torch.cuda.current_stream().cuda_stream
    xs = [torch.from_numpy(gen.to_nhwc_storage(b, "bf16").view(np.int16)).cuda() for b in batches]
    outs = [torch.empty((8, 1000), dtype=torch.float32, device="cuda:0") for _ in range(4)]
    worst = 0.0
    for _, members, bi in reqs:
        specs, keep = [], []
        for mi in members:
            m, blob, act, packed = pool[mi]
            s, k = fi.make_spec(m, packed.data_ptr(), packed.numel(), act_dtype=act, packed=True)
            specs.append(s)
            keep.append(k)
        dag = fi.Dag(specs, 8, alloc, keepalive=keep)
        dag.load(stream)
        for o in outs:
            o.fill_(float("nan"))
        dag.run(xs[bi].data_ptr(), 8, [o.data_ptr() for o in outs], stream)
        torch.cuda.synchronize()
        got = [o.cpu().numpy() for o in outs]
        dag.unload()
        dag.destroy()
        for slot, mi in enumerate(members):
            ref_f, ref_s = memo[(mi, bi)]
            y = got[slot][sample]
            wide = pool[mi][2] == "f32"
            worst = max(worst, harness.check_member(f"model {mi} batch {bi}", y, ref_f, ref_s, wide, quiet=True))
    assert not alloc.live or all(not t.is_cuda for t in alloc.live.values())  # nothing left on the device
    print(f"  {len(reqs)} requests replayed, worst member relL2 {worst:.3e}")
