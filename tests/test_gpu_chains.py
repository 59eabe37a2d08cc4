"""Chained convolutions (a dense convolution and the one or two pointwise convolutions behind it in one launch per
128-pixel tile: a bottleneck's 3x3, its 1x1 expansion with the shortcut added, the next block's 1x1 reduction).  The
chained schedule must equal, bit for bit, the schedule that launches every convolution by itself (Section III-A,
C1: the output of each model remains the same), and meet the oracle like it."""
import numpy as np
import pytest

from workloads import gen, zoo

pytestmark = pytest.mark.gpu


def _run(mem, x, **kw):
    from tests import harness
    g = harness.GpuDag(mem, x.shape[0], **kw)
    try:
        names = [L.name.decode() for L in g.dag.launches()]
        return g.run(x), names, g.dag.query()
    finally:
        g.close()


@pytest.mark.parametrize("fam,hw,batch", [("resnet50", 64, 5), ("resnet50", 96, 3), ("resnet101", 64, 2), ("wide_resnet50_2", 224, 2),
                                          ("resnet152", 32, 7)])
def test_chained_schedule_equals_separate_launches_bitwise(fam, hw, batch):
    from tests import harness
    mem = [(zoo.FAMILIES[fam](hw=hw), None, None) for _ in range(3)]
    mem = [(m, gen.make_blob(m, 4100 + i), None) for i, (m, _, _) in enumerate(mem)]
    x = gen.make_input(41, batch, 3, hw, hw, "normal", "bf16")
    fast, names, q = _run(mem, x)
    plain, pnames, pq = _run(mem, x, separate_chains=True)
    assert "conv_chain3" in names and not any(n.startswith("conv_chain") for n in pnames), (names, pnames)
    assert q.n_launches < pq.n_launches
    for i, (a, b) in enumerate(zip(fast, plain)):
        assert np.isfinite(a).all()
        assert np.array_equal(a, b), f"{fam} member {i}: the chained schedule differs from separate launches"
    m, blob, _ = mem[1]
    harness.check_against_oracle(f"{fam} (chained)", m, blob, None, x, fast[1])


def test_chains_next_to_other_members_and_under_every_build_option():
    """Chained members beside members that have no chain (VGG, MobileNetV2 with fp32 activations, a ResNet-18), in
    other slots, ungrouped, on one stream, as a HIP graph, with fewer images than max_batch: the same bits."""
    from tests import harness
    hw = 64
    fams = [("resnet50", None), ("vgg11", None), ("mobilenetv2", "f32"), ("resnet50", None), ("resnet18", None)]
    mem = []
    for i, (f, act) in enumerate(fams):
        m = zoo.FAMILIES[f](hw=hw)
        mem.append((m, gen.make_blob(m, 4200 + i), act))
    x = gen.make_input(43, 4, 3, hw, hw, "normal", "bf16")
    base, names, _ = _run(mem, x)
    assert "conv_chain3" in names
    for kw in (dict(separate_chains=True), dict(group_levels=False), dict(serial_lanes=True), dict(use_graph=True)):
        got, _, _ = _run(mem, x, **kw)
        for i, (a, b) in enumerate(zip(base, got)):
            assert np.array_equal(a, b), (kw, i)
    alone, _, _ = _run([mem[3]], x)
    assert np.array_equal(alone[0], base[3])
    order = [3, 2, 4, 0, 1]
    perm, _, _ = _run([mem[i] for i in order], x)
    for slot, i in enumerate(order):
        assert np.array_equal(perm[slot], base[i]), i
    from tests.harness import GpuDag
    g = GpuDag(mem, 9)   # room for 9 images: 9 given, then 4 (other ragged tiles in every stage); an image's bits do not depend on its batch
    try:
        x9 = np.concatenate([x, gen.make_input(44, 5, 3, hw, hw, "normal", "bf16")])
        full = g.run(x9)
        few = g.run(x)
    finally:
        g.close()
    for a, b in zip(few, full):
        assert np.array_equal(a, b[:4])
    for i in (0, 3):
        harness.check_against_oracle(f"resnet50[{i}] beside other members", mem[i][0], mem[i][1], None, x, base[i])


@pytest.mark.parametrize("chunks", [2, 3])
def test_member_chunks_keep_every_bit(chunks):
    """The early levels of a lane's members run chunk after chunk (a smaller activation arena, more launches): every
    member's output keeps its bits, next to lanes that have a single member."""
    from tests import harness
    hw = 96
    fams = [("resnet50", None)] * 5 + [("vgg11", None), ("mobilenetv2", "f32"), ("mobilenetv2", "f32"), ("densenet121", None), ("densenet121", None)]
    mem = []
    for i, (f, act) in enumerate(fams):
        m = zoo.FAMILIES[f](hw=hw)
        mem.append((m, gen.make_blob(m, 4300 + i), act))
    x = gen.make_input(45, 3, 3, hw, hw, "normal", "bf16")
    base, _, qb = _run(mem, x)
    got, _, qc = _run(mem, x, member_chunks=chunks)
    assert qc.act_bytes < qb.act_bytes and qc.n_launches > qb.n_launches
    for i, (a, b) in enumerate(zip(base, got)):
        assert np.isfinite(a).all() and np.array_equal(a, b), i
    serial, _, _ = _run(mem, x, member_chunks=chunks, serial_lanes=True)
    for i, (a, b) in enumerate(zip(base, serial)):
        assert np.array_equal(a, b), i
    harness.check_against_oracle("resnet50[4] in the last chunk", mem[4][0], mem[4][1], None, x, got[4])


def random_chain_model(seed):
    """A seeded random chain outside the bottleneck pattern (see the test below).  Returns (model, batch, description)."""
    import random
    rng = random.Random(9100 + seed)
    acts = [zoo.NONE, zoo.RELU, zoo.RELU6, zoo.HARDSWISH, zoo.SILU]
    cin = rng.choice([64, 128, 192, 256])
    w1 = rng.choice([64, 128])
    n2 = rng.choice([128, 256, 384, 512])
    n3 = rng.choice([0, 64, 128])
    kh, kw_ = rng.choice([(1, 1), (3, 3), (3, 3), (5, 5), (1, 3), (3, 1)])
    stride = rng.choice([1, 1, 2])
    same = max(kh, kw_) // 2
    pad = rng.choice([0, same])
    h, w = rng.randint(9, 23), rng.randint(9, 23)
    batch = rng.randint(1, 5)
    if kh * kw_ * cin >= 1024:   # a long reduction over few pixels would be split over K, and a split convolution heads no chain
        h, w = rng.randint(33, 47), rng.randint(33, 47)
        ho, wo = (h + 2 * pad * (kh > 1) - kh) // stride + 1, (w + 2 * pad * (kw_ > 1) - kw_) // stride + 1
        batch = -(-(130 * 64 // (w1 // 64)) // (ho * wo))
    m = zoo.Model(f"chain{seed}", "bf16", 16, h, w)
    x0 = m.add(zoo.CONV, -1, cin=16, cout=cin, k=3, stride=1, pad=1, act=zoo.RELU)
    x1 = m.add(zoo.CONV, x0, cin=cin, cout=cin, k=1, stride=1, pad=0, act=zoo.RELU)   # the chain's input: an intermediate tensor
    res = None
    if pad == same and rng.random() < 0.7:   # a residual of B's shape, one level above the chain: a strided 1x1 projection
        res = m.add(zoo.CONV, x0, cin=cin, cout=n2, k=1, stride=stride, pad=0, act=zoo.NONE)
    a = m.add(zoo.CONV, x1, cin=cin, cout=w1, k=kh, kw=(kw_ if kw_ != kh else 0), stride=stride, pad=pad, act=rng.choice(acts))
    b = m.add(zoo.CONV, a, cin=w1, cout=n2, k=1, stride=1, pad=0, act=rng.choice(acts), **({"residual": res} if res is not None else {}))
    tail = b
    if n3:
        tail = m.add(zoo.CONV, b, cin=n2, cout=n3, k=1, stride=1, pad=0, act=rng.choice(acts))
    both = m.add(zoo.CONV, tail, cin=(n3 or n2), cout=24, k=3, stride=1, pad=1, act=zoo.NONE)
    if n3:   # B's output has a second reader, as a block output has in a residual network
        m.add(zoo.CONV, b, cin=n2, cout=24, k=1, stride=1, pad=0, act=zoo.NONE, residual=both)
    m.shapes()
    return m, batch, f"{cin}->{w1} {kh}x{kw_}/{stride} pad {pad}, ->{n2} (residual {res is not None}), ->{n3}, image {h}x{w}, batch {batch}"


@pytest.mark.parametrize("seed", range(24))
def test_random_chains_equal_separate_launches_and_meet_the_oracle(seed):
    """Seeded random chains outside the bottleneck pattern: first convolutions of every kernel shape (1x1, 3x3, 5x5,
    rectangular, stride 2, with and without padding), 64 or 128 channels, second convolutions of 128 to 512 channels with
    and without a residual, with and without a third convolution, every activation, non-square images and batches
    whose pixel count leaves ragged tiles.  The model output is taken behind further convolutions so that every
    chained tensor is an intermediate one.  Chained = separate launches, bit for bit; both meet the oracle."""
    from tests import harness
    m, batch, what = random_chain_model(seed)
    blob = gen.make_blob(m, 9200 + seed)
    x = gen.make_input(9300 + seed, batch, 16, m.in_h, m.in_w, "normal", "bf16")
    print(f"seed {seed}: {what}", flush=True)
    fast, names, _ = _run([(m, blob, None)], x)
    plain, pnames, _ = _run([(m, blob, None)], x, separate_chains=True)
    assert any(n.startswith("conv_chain") for n in names), names
    assert not any(n.startswith("conv_chain") for n in pnames)
    assert np.isfinite(fast[0]).all() and np.array_equal(fast[0], plain[0])
    ref_f = harness.oracle_nhwc(m, blob, x, False)
    ref_s = harness.oracle_nhwc(m, blob, x, True)
    assert harness.rel_l2(fast[0], ref_f) <= 1e-2
    assert harness.elem_excess(fast[0], ref_s, harness.ELEM_C_BF16) <= 1.0
