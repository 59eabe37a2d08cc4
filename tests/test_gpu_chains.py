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
