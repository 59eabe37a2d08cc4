"""The stem launch: a 7x7 stride-2 (3x3 stride-1, 3x3 stride-2) convolution over the model input computed from an input
patch held on chip, a stride-2 one with the 3x3 stride-2 max-pool that alone reads it in the same launch (Section V,
Table III: the first layers of the ResNet-style families, of VGG, of SqueezeNet 1.1).  It must equal, bit for bit, the general convolution kernel followed by a pooling launch
(Section III-A, C1: the output of each model remains the same), and meet the oracle like them."""
import numpy as np
import pytest

from workloads import gen, zoo

pytestmark = pytest.mark.gpu


def stem_model(h, w, pad=3, pool="3x3/2", act=zoo.RELU, cout_tail=16, k=7, stride=2):
    """conv 7x7/2 -> [max-pool] -> 1x1 convolution whose fp32 output is the member's output: every pixel of the stem's
    tensor reaches the caller."""
    m = zoo.Model(f"stem{k}s{stride}_{h}x{w}p{pad}{pool}", "bf16", 3, h, w)
    a = m.add(zoo.CONV, zoo.MODEL_INPUT, cin=3, cout=64, k=k, stride=stride, pad=pad, act=act)
    if pool == "3x3/2":
        a = m.add(zoo.MAXPOOL, a, k=3, stride=2, pad=1)
    elif pool == "ceil":
        a = m.add(zoo.MAXPOOL, a, k=3, stride=2, pad=0, ceil=True)
    elif pool == "2x2/2":
        a = m.add(zoo.MAXPOOL, a, k=2, stride=2, pad=0)
    m.add(zoo.CONV, a, cin=64, cout=cout_tail, k=1, stride=1, pad=0, act=zoo.NONE)
    return m.shapes()


def _run(mem, x, **kw):
    from tests import harness
    g = harness.GpuDag(mem, x.shape[0], **kw)
    try:
        names = [L.name.decode() for L in g.dag.launches()]
        return g.run(x), names
    finally:
        g.close()


CASES = [
    # h, w, pad, pool, act, batch
    (224, 224, 3, "3x3/2", zoo.RELU, 2),     # the ImageNet stem: 56 x 56 pooled pixels are whole 7 x 8 blocks
    (64, 64, 3, "3x3/2", zoo.RELU, 5),
    (97, 131, 3, "3x3/2", zoo.RELU, 3),      # odd sizes: ragged blocks on both edges, a pool window hanging over the last row
    (33, 50, 3, "3x3/2", zoo.NONE, 4),       # no activation: negative values through the pool
    (17, 23, 3, "3x3/2", zoo.RELU6, 7),      # smaller than one block
    (230, 38, 0, "3x3/2", zoo.RELU, 2),      # no padding
    (75, 75, 1, "3x3/2", zoo.RELU, 3),
    (224, 224, 3, None, zoo.RELU, 2),        # no pool behind the convolution: the stem kernel alone
    (97, 131, 3, None, zoo.NONE, 3),
    (40, 29, 2, None, zoo.RELU6, 6),
    (112, 112, 3, "ceil", zoo.RELU, 3),      # ceil mode without padding (GoogLeNet): the last window hangs over the border
    (99, 61, 3, "ceil", zoo.NONE, 4),
    (224, 224, 3, "ceil", zoo.RELU, 2),
    (90, 90, 3, "2x2/2", zoo.RELU, 3),       # a pool the launch does not take: stem kernel + pooling launch
]


@pytest.mark.parametrize("h,w,pad,pool,act,batch", CASES)
def test_stem_launch_equals_general_kernels_bitwise_and_meets_the_oracle(h, w, pad, pool, act, batch):
    from tests import harness
    print(f"stem case {h}x{w} pad {pad} pool {pool} act {act} batch {batch}", flush=True)
    models = [stem_model(h, w, pad, pool, act) for _ in range(3)]
    mem = [(m, gen.make_blob(m, 5100 + i), None) for i, m in enumerate(models)]
    x = gen.make_input(51 + h, batch, 3, h, w, "normal", "bf16")
    fast, names = _run(mem, x)
    plain, pnames = _run(mem, x, separate_stem=True)
    want = "conv_stem_pool" if pool in ("3x3/2", "ceil") else "conv_stem"
    assert want in names and not any(n.startswith("conv_stem") for n in pnames), (names, pnames)
    if pool in ("3x3/2", "ceil"):
        assert "maxpool" not in names and "maxpool" in pnames
    for i, (a, b) in enumerate(zip(fast, plain)):
        assert np.isfinite(a).all()
        assert np.array_equal(a, b), f"member {i}: the stem launch differs from the general kernels"
    harness.check_against_oracle(f"stem {h}x{w} {pool}", mem[1][0], mem[1][1], None, x, fast[1])


SMALL_FILTER_CASES = [
    # k, stride, h, w, pad, pool, act, batch
    (3, 1, 224, 224, 1, None, zoo.RELU, 2),     # VGG's first layer
    (3, 1, 37, 53, 1, None, zoo.NONE, 3),       # ragged blocks
    (3, 1, 16, 16, 0, None, zoo.RELU6, 5),      # no padding, 14 x 14 outputs: less than a block
    (3, 1, 50, 21, 1, "2x2/2", zoo.RELU, 2),    # a pool behind a stride-1 layer keeps its launch
    (3, 2, 224, 224, 0, "ceil", zoo.RELU, 2),   # SqueezeNet 1.1's first two layers
    (3, 2, 95, 64, 1, "3x3/2", zoo.RELU, 3),
    (3, 2, 61, 77, 0, None, zoo.NONE, 4),
    (3, 2, 33, 20, 1, "ceil", zoo.RELU6, 6),
]


@pytest.mark.parametrize("k,stride,h,w,pad,pool,act,batch", SMALL_FILTER_CASES)
def test_small_filter_stems_equal_general_kernels_bitwise_and_meet_the_oracle(k, stride, h, w, pad, pool, act, batch):
    from tests import harness
    print(f"stem case {k}x{k}/{stride} {h}x{w} pad {pad} pool {pool} act {act} batch {batch}", flush=True)
    models = [stem_model(h, w, pad, pool, act, k=k, stride=stride) for _ in range(3)]
    mem = [(m, gen.make_blob(m, 5800 + i), None) for i, m in enumerate(models)]
    x = gen.make_input(59 + h, batch, 3, h, w, "normal", "bf16")
    fast, names = _run(mem, x)
    plain, pnames = _run(mem, x, separate_stem=True)
    fused = stride == 2 and pool in ("3x3/2", "ceil")
    assert ("conv_stem_pool" if fused else "conv_stem") in names and not any(n.startswith("conv_stem") for n in pnames), (names, pnames)
    assert ("maxpool" in names) == (pool is not None and not fused)
    for i, (a, b) in enumerate(zip(fast, plain)):
        assert np.isfinite(a).all()
        assert np.array_equal(a, b), f"member {i}: the stem launch differs from the general kernels"
    harness.check_against_oracle(f"stem {k}x{k}/{stride} {h}x{w} {pool}", mem[1][0], mem[1][1], None, x, fast[1])


@pytest.mark.parametrize("seed", range(24))
def test_random_stems_equal_general_kernels(seed):
    """Seeded random image sizes (1 to 5 blocks a side, every remainder), paddings, pools, activations and batches."""
    rng = np.random.default_rng(9000 + seed)
    k, stride = [(7, 2), (3, 1), (3, 2)][seed % 3]
    h, w = int(rng.integers(7, 150)), int(rng.integers(7, 150))
    pad = int(rng.integers(0, k // 2 + 1))
    pool = [None, "3x3/2", "ceil", "3x3/2"][int(rng.integers(0, 4))]
    act = [zoo.NONE, zoo.RELU, zoo.RELU6][int(rng.integers(0, 3))]
    batch = int(rng.integers(1, 6))
    if pool is not None and min((h + 2 * pad - k) // stride + 1, (w + 2 * pad - k) // stride + 1) < 3:
        pool = None   # (a pooling window larger than the tensor)
    print(f"random stem {seed}: {k}x{k}/{stride} {h}x{w} pad {pad} pool {pool} act {act} batch {batch}", flush=True)
    models = [stem_model(h, w, pad, pool, act, k=k, stride=stride) for _ in range(2)]
    mem = [(m, gen.make_blob(m, 5600 + 2 * seed + i), None) for i, m in enumerate(models)]
    x = gen.make_input(5700 + seed, batch, 3, h, w, "normal", "bf16")
    fast, names = _run(mem, x)
    plain, pnames = _run(mem, x, separate_stem=True)
    assert any(n.startswith("conv_stem") for n in names) and not any(n.startswith("conv_stem") for n in pnames)
    for a, b in zip(fast, plain):
        assert np.isfinite(a).all() and np.array_equal(a, b)
    from tests import harness
    harness.check_against_oracle(f"random stem {seed}", mem[0][0], mem[0][1], None, x, fast[0])


def test_stem_launch_under_every_build_option_and_beside_other_members():
    """ResNets (stem + pool in one launch) beside a VGG and an fp32-activation MobileNetV2 (general kernels), ungrouped,
    on one stream, as a HIP graph, in member chunks, alone, with fewer images than max_batch: the same bits."""
    from tests import harness
    hw = 64
    fams = [("resnet18", None), ("vgg11", None), ("mobilenetv2", "f32"), ("resnet50", None), ("resnet18", None)]
    mem = []
    for i, (f, act) in enumerate(fams):
        m = zoo.FAMILIES[f](hw=hw)
        mem.append((m, gen.make_blob(m, 5200 + i), act))
    x = gen.make_input(53, 4, 3, hw, hw, "normal", "bf16")
    base, names = _run(mem, x)
    assert "conv_stem_pool" in names
    for kw in (dict(separate_stem=True), dict(group_levels=False), dict(serial_lanes=True), dict(use_graph=True), dict(member_chunks=2),
               dict(separate_stem=True, separate_chains=True)):
        got, _ = _run(mem, x, **kw)
        for i, (a, b) in enumerate(zip(base, got)):
            assert np.array_equal(a, b), (kw, i)
    alone, _ = _run([mem[0]], x)
    assert np.array_equal(alone[0], base[0])
    g = harness.GpuDag(mem, 9)   # room for 9 images: 9 given, then 4; an image's bits do not depend on its batch
    try:
        x9 = np.concatenate([x, gen.make_input(54, 5, 3, hw, hw, "normal", "bf16")])
        full = g.run(x9)
        few = g.run(x)
    finally:
        g.close()
    for a, b in zip(few, full):
        assert np.array_equal(a, b[:4])
    for i in (0, 3):
        harness.check_against_oracle(f"{fams[i][0]} with the stem launch", mem[i][0], mem[i][1], None, x, base[i])


def test_stem_launch_writes_its_pooled_tensor_inside_a_concatenation():
    """The first tensor of a DenseNet block is stored inside the block's concatenation (no concat launch): the stem launch
    then writes its pooled pixels at that tensor's channel stride."""
    from tests import harness
    h, w, batch = 70, 52, 3
    m = zoo.Model("stem_concat", "bf16", 3, h, w)
    a = m.add(zoo.CONV, zoo.MODEL_INPUT, cin=3, cout=64, k=7, stride=2, pad=3, act=zoo.RELU)
    pool = m.add(zoo.MAXPOOL, a, k=3, stride=2, pad=1)
    b = m.add(zoo.DWCONV, pool, cin=64, cout=64, k=1, stride=1, pad=0, act=zoo.RELU, bn=False)   # (a dense layer: per-channel affine,
    b = m.add(zoo.CONV, b, cin=64, cout=128, k=1, stride=1, pad=0, act=zoo.RELU)                  # 1x1 squeeze, 3x3 with the new channels)
    b = m.add(zoo.CONV, b, cin=128, cout=32, k=3, stride=1, pad=1, act=zoo.NONE, bias=False, bn=False)
    c = m.add(zoo.CONCAT, pool, residual=b)
    m.add(zoo.CONV, c, cin=96, cout=24, k=1, stride=1, pad=0, act=zoo.NONE)
    m.shapes()
    mem = [(m, gen.make_blob(m, 5400 + i), None) for i in range(2)]
    x = gen.make_input(57, batch, 3, h, w, "normal", "bf16")
    fast, names = _run(mem, x)
    plain, pnames = _run(mem, x, separate_stem=True)
    copied, cnames = _run(mem, x, copy_concats=True)
    assert "conv_stem_pool" in names and "concat" not in names and "concat" in cnames and "conv_stem_pool" in cnames
    for a1, b1, c1 in zip(fast, plain, copied):
        assert np.isfinite(a1).all() and np.array_equal(a1, b1) and np.array_equal(a1, c1)
    harness.check_against_oracle("stem into a concatenation", m, mem[0][1], None, x, fast[0])
    # DenseNet-121: the same layout in a whole model
    dm = zoo.FAMILIES["densenet121"](hw=64)
    dmem = [(dm, gen.make_blob(dm, 5410 + i), None) for i in range(2)]
    dx = gen.make_input(58, 2, 3, 64, 64, "normal", "bf16")
    dfast, dnames = _run(dmem, dx)
    dplain, _ = _run(dmem, dx, separate_stem=True)
    assert "conv_stem_pool" in dnames
    for a1, b1 in zip(dfast, dplain):
        assert np.array_equal(a1, b1)


def test_stem_launch_full_size_batch32_equals_general_kernels():
    """The launch configuration the benchmark times: ResNet-50 stems at 224 x 224, batch 32, two members."""
    hw, batch = 224, 32
    models = [stem_model(hw, hw) for _ in range(2)]
    mem = [(m, gen.make_blob(m, 5300 + i), None) for i, m in enumerate(models)]
    x = gen.make_input(55, batch, 3, hw, hw, "normal", "bf16")
    fast, names = _run(mem, x)
    plain, _ = _run(mem, x, separate_stem=True)
    assert "conv_stem_pool" in names
    for a, b in zip(fast, plain):
        assert np.array_equal(a, b)
