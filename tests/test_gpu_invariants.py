"""Method invariants on the GPU (Section III-A C1/C4, Section IV-C): a member's output in a
fused DAG equals, bit for bit, the member run alone; changing or removing a co-member changes
no bit of it; permuting members permutes outputs; grouped and ungrouped schedules agree."""
import numpy as np
import pytest

from workloads import gen, zoo

pytestmark = pytest.mark.gpu


def _members(hw=64):
    fams = [("resnet18", None), ("mobilenetv2", None), ("vgg16", None), ("resnet50", None), ("mobilenetv2", "f32")]
    out = []
    for i, (f, act) in enumerate(fams):
        m = zoo.FAMILIES[f](hw=hw)
        out.append((m, gen.make_blob(m, 1000 + i), act))
    return out


def _run(mem, x, **kw):
    from tests import harness
    g = harness.GpuDag(mem, x.shape[0], **kw)
    try:
        return g.run(x)
    finally:
        g.close()


def test_fused_equals_alone_bitwise():
    mem = _members()
    x = gen.make_input(7, 3, 3, 64, 64, "normal", "bf16")
    fused = _run(mem, x)
    for i, mb in enumerate(mem):
        alone = _run([mb], x)[0]
        assert np.array_equal(fused[i], alone), f"member {i} differs from itself alone"


def test_isolation_and_permutation():
    mem = _members()
    x = gen.make_input(7, 2, 3, 64, 64, "normal", "bf16")
    base = _run(mem, x)
    # perturb member 1's weights: nobody else moves
    m1 = (mem[1][0], gen.make_blob(mem[1][0], 4242), mem[1][2])
    pert = _run([mem[0], m1] + mem[2:], x)
    for i in range(len(mem)):
        if i == 1:
            assert not np.array_equal(base[i], pert[i])
        else:
            assert np.array_equal(base[i], pert[i])
    # remove member 2
    less = _run(mem[:2] + mem[3:], x)
    assert all(np.array_equal(a, b) for a, b in zip(less, base[:2] + base[3:]))
    # permutation
    order = [3, 0, 4, 2, 1]
    perm = _run([mem[i] for i in order], x)
    for slot, i in enumerate(order):
        assert np.array_equal(perm[slot], base[i])


def test_grouped_equals_ungrouped_and_load_modes():
    import paper_2410_21120_amd as fi
    mem = _members()[:3]
    x = gen.make_input(7, 2, 3, 64, 64, "normal", "bf16")
    a = _run(mem, x, group_levels=True)
    b = _run(mem, x, group_levels=False)
    assert all(np.array_equal(u, v) for u, v in zip(a, b))
    # repository-time packing + per-model copies give the same bits as pack-at-build + one copy
    import torch
    packed = []
    for (m, blob, act) in mem:
        spec, keep = fi.make_spec(m, blob.ctypes.data, blob.nbytes, act_dtype=act)
        n = fi.fi_model_packed_size(spec)
        t = torch.empty(n, dtype=torch.uint8, pin_memory=True)
        fi.fi_model_pack(spec, t.data_ptr(), n)
        packed.append((m, t.numpy(), act))
    for mode in (fi.FI_LOAD_ONE_COPY, fi.FI_LOAD_PER_MODEL, fi.FI_LOAD_AUTO):
        c = _run(packed, x, load_mode=mode, packed=True)
        assert all(np.array_equal(u, v) for u, v in zip(a, c))
    # FI_LOAD_AUTO gathers only when it pays: members in device layout travel one by one on the first load of the handle,
    # as one image from the second load on; canonical members are packed at build, so their handle is one-copy from the start
    from tests import harness
    g = harness.GpuDag(packed, 2, load_mode=fi.FI_LOAD_AUTO, packed=True, swap_headroom_bytes=64 << 20)
    try:
        q = g.dag.query()
        assert (q.n_h2d_copies, q.last_h2d_copies) == (1 + len(packed), 1 + len(packed)) and q.last_h2d_bytes >= q.arena_bytes - 256 * len(packed)
        assert all(np.array_equal(u, v) for u, v in zip(a, g.run(x)))
        g.dag.unload()
        g.dag.load(g.stream)
        q = g.dag.query()
        assert (q.n_h2d_copies, q.last_h2d_copies, q.last_h2d_bytes) == (1, 1, q.arena_bytes)
        assert all(np.array_equal(u, v) for u, v in zip(a, g.run(x)))
        # a member swap on the gathered handle keeps the image exact: unload, load, same bits
        newcomer = (mem[1][0], gen.make_blob(mem[1][0], 4321), mem[1][2])
        g.packed = False
        g.swap(1, newcomer)
        after = g.run(x)
        g.dag.unload()
        g.dag.load(g.stream)
        assert all(np.array_equal(u, v) for u, v in zip(after, g.run(x)))
        assert np.array_equal(after[0], a[0]) and not np.array_equal(after[1], a[1])
    finally:
        g.close()
    g = harness.GpuDag(mem, 2, load_mode=fi.FI_LOAD_AUTO)
    try:
        q = g.dag.query()
        assert (q.n_h2d_copies, q.last_h2d_copies, q.last_h2d_bytes) == (1, 1, q.arena_bytes)
        assert all(np.array_equal(u, v) for u, v in zip(a, g.run(x)))
    finally:
        g.close()


def test_launch_counts_and_single_allocation():
    from tests import harness
    ms = []
    for i in range(4):
        m = zoo.resnet50(hw=64)
        ms.append((m, gen.make_blob(m, 1000 + i), None))
    g = harness.GpuDag(ms, 2)
    try:
        q = g.dag.query()
        assert q.n_device_allocs == 1 and q.n_h2d_copies == 1 and q.state == 1
        assert g.alloc.n_dev == 1 and g.alloc.n_pin == 1
        assert q.n_nodes == 4 * 56 and q.n_levels == 52
        # staging + one grouped launch per level (one more where members' shapes pick different tiles); a chained launch
        # stands for two or three levels
        main = [L for L in g.dag.launches() if L.name != b"splitk_reduce"]  # split-K launches add a reduce twin
        chained = sum(2 if L.name == b"conv_chain3" else 1 if L.name == b"conv_chain2" else 0 for L in main)
        assert 53 <= len(main) + chained <= 57 + 52
    finally:
        g.close()


def test_hip_graph_replay_matches_eager():
    """The schedule replayed as one HIP graph gives the eager bits on every replay, with other GPU work and
    synchronisations between replays, after a batch change (re-capture) and after new input values."""
    import torch
    from tests import harness
    mem = _members()[:3]
    x1 = gen.make_input(7, 3, 3, 64, 64, "normal", "bf16")
    x2 = gen.make_input(8, 3, 3, 64, 64, "normal", "bf16")
    eager1, eager2 = _run(mem, x1), _run(mem, x2)
    e = harness.GpuDag(mem, 3)  # same max_batch as the graph DAG: split-K factors are fixed at build time
    try:
        eager_small = e.run(x1[:2])
    finally:
        e.close()
    g = harness.GpuDag(mem, 3, use_graph=True)
    try:
        for rep in range(4):
            x, ref = (x1, eager1) if rep % 2 == 0 else (x2, eager2)
            got = g.run(x)  # same device buffers every time: replays after the first capture
            assert all(np.array_equal(a, b) for a, b in zip(got, ref)), f"replay {rep} differs"
            junk = torch.randn(1 << 20, device="cuda:0")  # unrelated eager work between replays
            (junk * 2).sum().item()
            torch.cuda.synchronize()
        small = g.run(x1[:2])  # other batch: the graph is rebuilt
        assert all(np.array_equal(a, b) for a, b in zip(small, eager_small))
        again = g.run(x1[:2])
        assert all(np.array_equal(a, b) for a, b in zip(again, eager_small))
    finally:
        g.close()


def test_concurrent_lanes_equal_serial_schedule():
    """Members of different architecture run on concurrent internal streams; the bits are those of the
    single-stream schedule, run after run."""
    mem = _members()
    x = gen.make_input(7, 3, 3, 64, 64, "normal", "bf16")
    serial = _run(mem, x, serial_lanes=True)
    from tests import harness
    g = harness.GpuDag(mem, 3)
    try:
        assert g.dag.query().n_lanes == 5
        for _ in range(3):
            got = g.run(x)
            assert all(np.array_equal(a, b) for a, b in zip(got, serial))
    finally:
        g.close()


def test_timeline_pass_gives_the_same_bits_and_ordered_intervals():
    """The timed pass is the ordinary pass plus events: same outputs; on every lane the launches follow
    each other (a launch begins where the previous one on its stream ended), the input staging precedes
    everything, and no interval is empty or reversed."""
    mem = _members()
    x = gen.make_input(7, 3, 3, 64, 64, "normal", "bf16")
    from tests import harness
    g = harness.GpuDag(mem, 3)
    try:
        ref = g.run(x)
        got, (tb, te) = g.run(x, profile="timeline")
        assert all(np.array_equal(a, b) for a, b in zip(got, ref))
        launches = g.dag.launches()
        assert len(tb) == len(te) == len(launches)
        last_end = {}
        stage_end = max(e for L, e in zip(launches, te) if L.level == 0)
        for L, b, e in zip(launches, tb, te):
            assert 0.0 <= b <= e
            if L.level > 0:
                assert b >= stage_end - 1e-3
                assert b >= last_end.get(L.lane, 0.0) - 1e-3  # issue order on a stream is execution order
                last_end[L.lane] = e
        assert len(last_end) == g.dag.query().n_lanes
    finally:
        g.close()


def test_per_member_inputs_equal_each_member_alone_on_its_input():
    """Algorithm 1 feeds every member model its own input: member m of a DAG built for per-member inputs,
    given input m, produces the bits of member m alone on that input; one pointer for all of them gives
    the bits of the shared-input DAG."""
    import torch
    import paper_2410_21120_amd as fi
    from tests import harness
    mem = _members()
    xs = [gen.make_input(20 + i, 3, 3, 64, 64, "normal", "bf16") for i in range(len(mem))]
    alone = [_run([mb], x)[0] for mb, x in zip(mem, xs)]
    shared = _run(mem, xs[0])
    specs, keep = [], []
    for m, blob, act in mem:
        sp, k = fi.make_spec(m, blob.ctypes.data, blob.nbytes, act_dtype=act)
        specs.append(sp)
        keep.append((k, blob))
    alloc = fi.TorchAllocators("cuda:0")
    dag = fi.Dag(specs, 3, alloc, keepalive=keep, per_member_inputs=True)
    stream = torch.cuda.current_stream().cuda_stream
    dag.load(stream)
    try:
        dev_in = [torch.from_numpy(gen.to_nhwc_storage(x, "bf16").view(np.int16)).cuda() for x in xs]
        outs = [torch.full((3, 1000), float("nan"), dtype=torch.float32, device="cuda:0") for _ in mem]
        assert dag.query().n_lanes == 5
        for _ in range(2):
            dag.run_inputs([t.data_ptr() for t in dev_in], 3, [o.data_ptr() for o in outs], stream)
            torch.cuda.synchronize()
            for i, o in enumerate(outs):
                assert np.array_equal(o.cpu().numpy(), alone[i]), f"member {i}"
        dag.run(dev_in[0].data_ptr(), 3, [o.data_ptr() for o in outs], stream)
        torch.cuda.synchronize()
        for i, o in enumerate(outs):
            assert np.array_equal(o.cpu().numpy(), shared[i])
    finally:
        dag.unload()
        dag.destroy()
    # a DAG built for a shared input refuses per-member inputs
    g = harness.GpuDag(mem[:2], 3)
    try:
        with pytest.raises(fi.FiError) as e:
            g.dag.run_inputs([dev_in[0].data_ptr()] * 2, 3, [outs[0].data_ptr(), outs[1].data_ptr()], g.stream)
        assert e.value.status == fi.FI_ESTATE
    finally:
        g.close()


def test_run_time_argument_errors_on_a_loaded_dag():
    """Empty and oversized batches and missing buffers are refused before any launch; the DAG keeps working."""
    import ctypes as C
    import paper_2410_21120_amd as fi
    from tests import harness
    mem = _members()[:2]
    x = gen.make_input(7, 3, 3, 64, 64, "normal", "bf16")
    g = harness.GpuDag(mem, 3)
    try:
        base = g.run(x)
        b, xin, outs = g.keep_buffers
        ptrs = [o.data_ptr() for o in outs]
        for bad_batch in (0, -1, 4):
            with pytest.raises(fi.FiError) as e:
                g.dag.run(xin.data_ptr(), bad_batch, ptrs, g.stream)
            assert e.value.status == fi.FI_EINVAL
        with pytest.raises(fi.FiError) as e:
            g.dag.run(xin.data_ptr(), 3, [ptrs[0], 0], g.stream)
        assert e.value.status == fi.FI_EINVAL
        with pytest.raises(fi.FiError) as e:
            g.dag.run(0, 3, ptrs, g.stream)
        assert e.value.status == fi.FI_EINVAL
        with pytest.raises(fi.FiError) as e:
            g.dag.load(g.stream)                      # already loaded
        assert e.value.status == fi.FI_ESTATE
        assert all(np.array_equal(a, b2) for a, b2 in zip(g.run(x), base))
        assert all(np.array_equal(a[:1], b2) for a, b2 in zip(base, g.run(x[:1])))   # batch 1 of max 3: rows are independent
    finally:
        g.close()


def test_members_that_stage_the_input_differently():
    """An RGB-like input is staged with 4 channels for members whose input feeds only convolutions and with 8
    for the others (here: a pooling-first and a depthwise-first member): one DAG holds both copies and every
    member reads its own."""
    from tests import harness
    from workloads import zoo

    def member(first):
        m = zoo.Model(first, "bf16", 3, 20, 24)
        cur = -1
        if first == "pool":
            cur = m.add(zoo.MAXPOOL, cur, k=2, stride=2, pad=0)
        elif first == "dw":
            cur = m.add(zoo.DWCONV, cur, cin=3, cout=3, k=3, stride=1, pad=1, act=zoo.RELU)
        cur = m.add(zoo.CONV, cur, cin=3, cout=16, k=3, stride=1, pad=1, act=zoo.RELU)
        cur = m.add(zoo.GAP, cur)
        m.add(zoo.FC, cur, cin=16, cout=10)
        return m.shapes()
    for order in (["conv", "pool", "dw"], ["pool", "conv", "dw"]):
        models = [member(f) for f in order]
        blobs = [gen.make_blob(m, 40 + i) for i, m in enumerate(models)]
        x = gen.make_input(3, 3, 3, 20, 24, "normal", "bf16")
        g = harness.GpuDag([(m, b, "f32" if i == 2 else None) for i, (m, b) in enumerate(zip(models, blobs))], 3)
        try:
            ys = g.run(x)
        finally:
            g.close()
        for i, (m, b, y) in enumerate(zip(models, blobs, ys)):
            ref = harness.oracle_nhwc(m, b, x, False)
            assert harness.rel_l2(y, ref) <= (1e-4 if i == 2 else 1e-2), (order, i)


def _folded_members(hw=64):
    """Members whose schedules fold nodes: concatenations in place, absorbed affine nodes and scalings, group walks,
    interleaving shuffles; two of them of one architecture (grouped launches)."""
    fams = ["densenet121", "googlenet", "mobilenet_v3_small", "shufflenet_v2_x1_0", "densenet121"]
    out = []
    for i, f in enumerate(fams):
        m = zoo.FAMILIES[f](hw=hw)
        out.append((m, gen.make_blob(m, 1200 + i), None))
    return out


@pytest.mark.parametrize("members", ["classic", "folded"])
def test_per_member_batches(members):
    """The manager aggregates requests per model, so members arrive at a pass with different numbers of images:
    member m on batches[m] images gives, bit for bit, what the same DAG gives for those images at the full
    batch; a member with no image sits the pass out and its output buffer is not touched."""
    import torch
    import paper_2410_21120_amd as fi
    mem = _members() if members == "classic" else _folded_members()
    B = 5
    xs = [gen.make_input(80 + i, B, 3, 64, 64, "normal", "bf16") for i in range(len(mem))]
    specs, keep = [], []
    for m, blob, act in mem:
        sp, k = fi.make_spec(m, blob.ctypes.data, blob.nbytes, act_dtype=act)
        specs.append(sp)
        keep.append((k, blob))
    dag = fi.Dag(specs, B, fi.TorchAllocators("cuda:0"), keepalive=keep, per_member_inputs=True)
    stream = torch.cuda.current_stream().cuda_stream
    dag.load(stream)
    try:
        dev_in = [torch.from_numpy(gen.to_nhwc_storage(x, "bf16").view(np.int16)).cuda() for x in xs]
        full = [torch.full((B, 1000), float("nan"), dtype=torch.float32, device="cuda:0") for _ in mem]
        dag.run_inputs([t.data_ptr() for t in dev_in], B, [o.data_ptr() for o in full], stream)
        torch.cuda.synchronize()
        full = [o.cpu().numpy() for o in full]
        for batches in ([5, 1, 0, 3, 2], [0, 0, 4, 0, 0], [1, 5, 5, 0, 5]):
            outs = [torch.full((B, 1000), -7.0, dtype=torch.float32, device="cuda:0") for _ in mem]
            ins = [t.data_ptr() if b else 0 for t, b in zip(dev_in, batches)]
            ops = [o.data_ptr() if b else 0 for o, b in zip(outs, batches)]
            dag.run_batches(ins, batches, ops, stream)
            torch.cuda.synchronize()
            for i, (o, b) in enumerate(zip(outs, batches)):
                y = o.cpu().numpy()
                assert np.array_equal(y[:b], full[i][:b]), (batches, i)
                assert np.all(y[b:] == -7.0), (batches, i)   # rows past the member's batch stay as they were
                # unequal batches, every member on an input of its own: against the oracle (all but the MobileNetV2
                # that stores bf16 activations, which no executor holds to the bar with these weights)
                if b and batches[0] == 5 and not (mem[i][0].name.startswith("mobilenetv2") and mem[i][2] is None):
                    from tests import harness
                    harness.check_against_oracle(f"member {i} on {b} of its own images", mem[i][0], mem[i][1], mem[i][2], xs[i][:b], y[:b])
        with pytest.raises(fi.FiError) as e:
            dag.run_batches([t.data_ptr() for t in dev_in], [B + 1, 1, 1, 1, 1], [o.data_ptr() for o in outs], stream)
        assert e.value.status == fi.FI_EINVAL
        with pytest.raises(fi.FiError) as e:
            dag.run_batches([0] + [t.data_ptr() for t in dev_in[1:]], [1, 1, 1, 1, 1], [o.data_ptr() for o in outs], stream)
        assert e.value.status == fi.FI_EINVAL
    finally:
        dag.unload()
        dag.destroy()


@pytest.mark.parametrize("members", ["classic", "folded"])
def test_lanes_run_alone_and_side_by_side(members):
    """fi_run_lane issues one lane of the schedule on the caller's stream: every lane on a stream of its own, all
    in flight together, gives each member the bits of the whole-DAG pass; a lane run alone leaves the members of
    the other lanes untouched."""
    import torch
    import paper_2410_21120_amd as fi
    if members == "classic":
        mem = _members()   # five architectures: five lanes
        mem = mem + [(mem[0][0], gen.make_blob(mem[0][0], 2222), None)]   # and a second ResNet-18 that shares lane 0
    else:
        mem = _folded_members()   # four architectures, the last member shares lane 0 with the first
    n_arch = len(mem) - 1
    B = 3
    xs = [gen.make_input(90 + i, B, 3, 64, 64, "normal", "bf16") for i in range(len(mem))]
    specs, keep = [], []
    for m, blob, act in mem:
        sp, k = fi.make_spec(m, blob.ctypes.data, blob.nbytes, act_dtype=act)
        specs.append(sp)
        keep.append((k, blob))
    dag = fi.Dag(specs, B, fi.TorchAllocators("cuda:0"), keepalive=keep, per_member_inputs=True)
    stream = torch.cuda.current_stream().cuda_stream
    dag.load(stream)
    try:
        q = dag.query()
        lane_of = [mi.lane for mi in dag.members()]
        assert q.n_lanes == n_arch and lane_of[0] == lane_of[-1] and len(set(lane_of)) == n_arch
        dev_in = [torch.from_numpy(gen.to_nhwc_storage(x, "bf16").view(np.int16)).cuda() for x in xs]
        batches = [3, 2, 1, 3, 2, 1][:len(mem) - 1] + [1]
        ref = [torch.full((B, 1000), -3.0, dtype=torch.float32, device="cuda:0") for _ in mem]
        dag.run_batches([t.data_ptr() for t in dev_in], batches, [o.data_ptr() for o in ref], stream)
        torch.cuda.synchronize()
        ref = [o.cpu().numpy() for o in ref]
        # one lane alone
        outs = [torch.full((B, 1000), -3.0, dtype=torch.float32, device="cuda:0") for _ in mem]
        torch.cuda.synchronize()
        dag.run_lane(lane_of[0], [t.data_ptr() for t in dev_in], batches, [o.data_ptr() for o in outs], stream)
        torch.cuda.synchronize()
        for i, o in enumerate(outs):
            y = o.cpu().numpy()
            if lane_of[i] == lane_of[0]:
                assert np.array_equal(y, ref[i]), i
            else:
                assert np.all(y == -3.0), i
        # every lane on its own stream, all issued before any is waited for, three times over
        streams = [torch.cuda.Stream() for _ in range(q.n_lanes)]
        for _ in range(3):
            outs = [torch.full((B, 1000), -3.0, dtype=torch.float32, device="cuda:0") for _ in mem]
            torch.cuda.synchronize()
            for lane, st in enumerate(streams):
                dag.run_lane(lane, [t.data_ptr() for t in dev_in], batches, [o.data_ptr() for o in outs], st.cuda_stream)
            torch.cuda.synchronize()
            for i, o in enumerate(outs):
                assert np.array_equal(o.cpu().numpy(), ref[i]), i
        with pytest.raises(fi.FiError) as e:
            dag.run_lane(q.n_lanes, [t.data_ptr() for t in dev_in], batches, [o.data_ptr() for o in outs], stream)
        assert e.value.status == fi.FI_EINVAL
    finally:
        dag.unload()
        dag.destroy()


@pytest.mark.parametrize("fam", ["densenet121", "googlenet", "squeezenet1_0", "inception_v3", "shufflenet_v2_x0_5", "shufflenet_v2_x1_0"])
def test_concatenations_in_place_equal_copied_ones(fam):
    """Sources written straight into the concatenation's tensor (dense blocks, Inception and fire modules, the kept half
    of a shuffle unit) against a handle that copies at every concatenation and launches every absorbed node: fewer
    launches, the same bits, also at a batch below the planned one and with two members sharing launches."""
    from tests import harness
    hw = 96 if fam == "inception_v3" else 64
    m = zoo.FAMILIES[fam](hw=hw)
    blobs = [gen.make_blob(m, 300 + i) for i in range(2)]
    x = gen.make_input(11, 3, 3, hw, hw, "normal", "bf16")
    res, launches = {}, {}
    for copy in (False, True):
        g = harness.GpuDag([(m, b, None) for b in blobs], 3, copy_concats=copy, separate_affine=copy)
        try:
            launches[copy] = g.dag.query().n_launches
            names = [L.name.decode() for L in g.dag.launches()]
            res[copy] = [g.run(x), g.run(x[:2])]
        finally:
            g.close()
        # (the 58-channel halves of x1.0 are not vector aligned and cannot be stored in place: there the two-group shuffle
        # that follows every concatenation interleaves the halves itself)
        assert ("concat" in names) == copy
    assert launches[False] < launches[True]
    for r0, r1 in zip(res[False], res[True]):
        for y0, y1 in zip(r0, r1):
            assert np.isfinite(y0).all() and np.array_equal(y0, y1)


def _dense_block(c0, growth, layers, h, w):
    m = zoo.Model("dense", "bf16", 8, h, w)
    t = m.add(zoo.CONV, -1, cin=8, cout=c0, k=3, stride=1, pad=1, act=zoo.RELU)
    c = c0
    for _ in range(layers):
        a = m.add(zoo.DWCONV, t, cin=c, cout=c, k=1, stride=1, pad=0, act=zoo.RELU)
        a = m.add(zoo.CONV, a, cin=c, cout=4 * growth, k=1, stride=1, pad=0, act=zoo.RELU)
        a = m.add(zoo.CONV, a, cin=4 * growth, cout=growth, k=3, stride=1, pad=1, act=zoo.NONE)
        t = m.add(zoo.CONCAT, t, residual=a)
        c += growth
    t = m.add(zoo.DWCONV, t, cin=c, cout=c, k=1, stride=1, pad=0, act=zoo.RELU6)     # a transition: affine, 1x1 convolution, pooling
    t = m.add(zoo.CONV, t, cin=c, cout=c // 2, k=1, stride=1, pad=0, act=zoo.NONE)
    t = m.add(zoo.AVGPOOL, t, k=2, stride=2, pad=0)
    t = m.add(zoo.GAP, t)
    m.add(zoo.FC, t, cin=c // 2, cout=10)
    return m.shapes()


@pytest.mark.parametrize("case", ["densenet121", "densenet161", "mobilenet_v3_large", "mobilenet_v3_small", "mobilenet_v3_large:f32", (16, 8, 3, 9, 7), (64, 32, 5, 28, 28),
                                  (24, 16, 2, 6, 6), (200, 40, 2, 14, 14)])
def test_affine_applied_by_the_convolution_equals_its_own_launch(case):
    """The per-channel affine + ReLU in front of a dense layer's 1x1 convolution, applied by that convolution while it
    loads its input (no launch, no tensor) against a handle that runs it as a depthwise launch: fewer launches, the
    same bits -- whole DenseNets and blocks whose channel counts leave ragged reduction tiles, split reductions and
    inputs inside a concatenation's tensor; also with copied concatenations (the input then has its own stride).  The
    MobileNetV3s cover the other absorbed node: the squeeze-excite scaling applied by the block's projection."""
    from tests import harness
    act = None
    if isinstance(case, str):
        fam, _, act = case.partition(":")   # "family:f32": fp32-stored activations (the scaling is absorbed there too)
        act = act or None
        m, hw = zoo.FAMILIES[fam](hw=64), (64, 64)
    else:
        m, hw = _dense_block(*case), case[3:]
    blobs = [gen.make_blob(m, 400 + i) for i in range(2)]
    x = gen.make_input(12, 3, m.in_c, hw[0], hw[1], "normal", "bf16")
    res, launches = {}, {}
    for key, kw in (("fused", {}), ("separate", dict(separate_affine=True)), ("fused_copy", dict(copy_concats=True)),
                    ("plain", dict(separate_affine=True, copy_concats=True))):
        g = harness.GpuDag([(m, b, act) for b in blobs], 3, **kw)
        try:
            launches[key] = g.dag.query().n_launches
            res[key] = [g.run(x), g.run(x[:1])]
        finally:
            g.close()
    assert launches["fused"] < launches["separate"] <= launches["plain"] and launches["fused_copy"] < launches["plain"]
    for key in ("separate", "fused_copy", "plain"):
        for r0, r1 in zip(res["fused"], res[key]):
            for y0, y1 in zip(r0, r1):
                assert np.isfinite(y0).all() and np.array_equal(y0, y1), key
