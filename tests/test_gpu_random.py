"""GPU parity on seeded random layer graphs: every operator in arbitrary order, odd channel counts, non-square
inputs, residuals and concatenations across distant nodes.  Each case fuses three random graphs that share the
input shape (two with bf16-stored activations, one with fp32-stored ones) into one DAG and compares every member
with the CPU oracle run on that member alone."""
import numpy as np
import pytest

from workloads import gen, randnet

pytestmark = pytest.mark.gpu

BF16_TOL = 1e-2   # relative L2 vs the fp32-activation oracle (mode F)
WIDE_TOL = 1e-4   # fp32-stored activations


@pytest.mark.parametrize("seed", range(0, 120, 3))
def test_three_random_graphs_fused(seed):
    from tests import harness
    first = randnet.random_model(seed)
    models = [first] + [randnet.random_model(seed + j, in_c=first.in_c, hw=(first.in_h, first.in_w)) for j in (1, 2)]
    batch = 1 + seed % 4
    blobs = [gen.make_blob(m, 7000 + seed + i) for i, m in enumerate(models)]
    x = gen.make_input(31 + seed, batch, first.in_c, first.in_h, first.in_w, "normal", "bf16")
    print(f"seed {seed}: batch {batch}, input {first.in_c}x{first.in_h}x{first.in_w}, nodes {[len(m.layers) for m in models]}", flush=True)
    g = harness.GpuDag([(models[0], blobs[0], None), (models[1], blobs[1], None), (models[2], blobs[2], "f32")], batch)
    try:
        ys = g.run(x)
    finally:
        g.close()
    for i, (m, blob, y) in enumerate(zip(models, blobs, ys)):
        ref_f = harness.oracle_nhwc(m, blob, x, False)
        assert y.shape == ref_f.shape and np.isfinite(y).all()
        scale = max(float(np.linalg.norm(ref_f)), 1e-30)
        floor = 1e-5 * np.sqrt(ref_f.size) / scale   # outputs that are (nearly) all zero: absolute error of 1e-5 per element
        e_f = harness.rel_l2(y, ref_f)
        if i == 2:
            assert e_f <= WIDE_TOL + floor, f"member {i} (fp32 activations): rel L2 {e_f}"
            continue
        # bf16-stored activations.  The oracle that rounds every stored tensor to bf16 (mode S) differs from the
        # library only by summation order and the rounding flips that causes; how far such flips travel is a
        # property of the graph, measured by the distance between the oracle's own two modes.
        ref_s = harness.oracle_nhwc(m, blob, x, True)
        d_sf = harness.rel_l2(ref_s, ref_f)
        e_s = harness.rel_l2(y, ref_s)
        assert e_s <= max(2e-3, 0.5 * d_sf) + floor, f"member {i}: rel L2 vs storage-rounding oracle {e_s}, modes differ by {d_sf}"
        if d_sf <= 0.5 * BF16_TOL:   # graphs on which bf16 storage itself stays inside the bar
            assert e_f <= BF16_TOL + floor, f"member {i}: rel L2 {e_f}"


@pytest.mark.parametrize("seed", range(1, 120, 6))
def test_random_graphs_keep_their_bits_under_every_build_option(seed):
    """The invariants of the method on random graphs: a member's output is the same, bit for bit, alone, next to
    other members, in another slot, ungrouped, on one stream, replayed as a HIP graph, loaded from device-layout
    blobs with one copy per member, with fewer images in the batch, given its input through the
    per-member entry point, and after its neighbour was swapped for another model."""
    import torch
    import paper_2410_21120_amd as fi
    from tests import harness
    first = randnet.random_model(seed)
    same = dict(in_c=first.in_c, hw=(first.in_h, first.in_w))
    models = [first, randnet.random_model(seed + 1, **same), randnet.random_model(seed + 2, **same), first]
    acts = [None, "f32", None, None]   # members 0 and 3 share an architecture (one lane, grouped launches)
    batch = 2 + seed % 3
    mem = [(m, gen.make_blob(m, 9000 + seed + i), a) for i, (m, a) in enumerate(zip(models, acts))]
    x = gen.make_input(51 + seed, batch, first.in_c, first.in_h, first.in_w, "normal", "bf16")
    print(f"seed {seed}: batch {batch}, input {first.in_c}x{first.in_h}x{first.in_w}, nodes {[len(m.layers) for m in models]}", flush=True)

    def run(members, xx, **kw):
        g = harness.GpuDag(members, kw.pop("max_batch", xx.shape[0]), **kw)
        try:
            return g.run(xx)
        finally:
            g.close()
    base = run(mem, x)
    assert all(np.isfinite(y).all() for y in base)
    for i, mb in enumerate(mem):
        assert np.array_equal(run([mb], x)[0], base[i]), f"member {i} alone"
    order = [2, 3, 0, 1]
    for slot, y in zip(order, run([mem[i] for i in order], x)):
        assert np.array_equal(y, base[slot]), f"member {slot} permuted"
    packed = []   # repository-time device-layout blobs in pinned memory
    for m, blob, act in mem:
        spec, keep_spec = fi.make_spec(m, blob.ctypes.data, blob.nbytes, act_dtype=act)
        n = fi.fi_model_packed_size(spec)
        t = torch.empty(n, dtype=torch.uint8, pin_memory=True)
        fi.fi_model_pack(spec, t.data_ptr(), n)
        packed.append((m, t.numpy(), act))
    variants = dict(ungrouped=(mem, dict(group_levels=False)), serial=(mem, dict(serial_lanes=True)), graph=(mem, dict(use_graph=True)),
                    per_model_copies=(packed, dict(packed=True, load_mode=fi.FI_LOAD_PER_MODEL)),
                    packed_one_copy=(packed, dict(packed=True)),
                    # concatenations copied instead of written in place, affine nodes as launches of their own
                    copied_concats=(mem, dict(copy_concats=True)), separate_affine=(mem, dict(separate_affine=True)),
                    plain=(mem, dict(copy_concats=True, separate_affine=True, group_levels=False)))
    for name, (members, kw) in variants.items():
        for i, y in enumerate(run(members, x, **kw)):
            assert np.array_equal(y, base[i]), f"{name}: member {i}"
    # a DAG built for a larger batch: an image's output does not depend on how many images accompany it
    # (the split factors, and with them the summation order, belong to the DAG's max_batch, so the comparison
    # stays inside one DAG)
    more = np.concatenate([x, gen.make_input(52 + seed, 3, first.in_c, first.in_h, first.in_w, "normal", "bf16")])
    g = harness.GpuDag(mem, batch + 3)
    try:
        full, part = g.run(more), g.run(x)
    finally:
        g.close()
    for i in range(4):
        assert np.array_equal(full[i][:batch], part[i]), f"member {i} at a smaller batch"
    # per-member inputs: member i on input i equals member i alone on input i
    xs = [gen.make_input(60 + seed + i, batch, first.in_c, first.in_h, first.in_w, "normal", "bf16") for i in range(4)]
    alone = [run([mb], xi)[0] for mb, xi in zip(mem, xs)]
    specs, keep = [], []
    for m, blob, act in mem:
        sp, k = fi.make_spec(m, blob.ctypes.data, blob.nbytes, act_dtype=act)
        specs.append(sp)
        keep.append((k, blob))
    dag = fi.Dag(specs, batch, fi.TorchAllocators("cuda:0"), keepalive=keep, per_member_inputs=True)
    stream = torch.cuda.current_stream().cuda_stream
    dag.load(stream)
    try:
        dev_in = [torch.from_numpy(gen.to_nhwc_storage(xi, "bf16").view(np.int16)).cuda() for xi in xs]
        outs = [torch.full((batch, y.shape[1]), float("nan"), dtype=torch.float32, device="cuda:0") for y in base]
        dag.run_inputs([t.data_ptr() for t in dev_in], batch, [o.data_ptr() for o in outs], stream)
        torch.cuda.synchronize()
        for i, o in enumerate(outs):
            assert np.array_equal(o.cpu().numpy(), alone[i]), f"per-member input {i}"
    finally:
        dag.unload()
        dag.destroy()
    # swap member 1 for a fresh model: the others keep their bits, the newcomer equals itself alone
    fresh = randnet.random_model(seed + 7, **same)
    newcomer = (fresh, gen.make_blob(fresh, 9900 + seed), None)
    g = harness.GpuDag(mem, batch, swap_headroom_bytes=64 << 20)
    try:
        assert all(np.array_equal(a, b) for a, b in zip(g.run(x), base))
        g.swap(1, newcomer)
        after = g.run(x)
    finally:
        g.close()
    for i in (0, 2, 3):
        assert np.array_equal(after[i], base[i]), f"member {i} after its neighbour was swapped"
    assert np.array_equal(after[1], run([newcomer], x)[0])


@pytest.mark.parametrize("seed", range(200, 214))
def test_large_random_graphs_fused(seed):
    """Random graphs on tensors large enough for the big convolution tiles (40-90 pixels a side, up to 512
    channels, batch 6): two members of one architecture with bf16-stored activations (one grouped launch per
    level) and a third with fp32-stored ones, each against the oracle on that member alone."""
    from tests import harness
    m = randnet.random_model(seed, large=True, max_nodes=8)
    batch = 6
    blobs = [gen.make_blob(m, 8000 + seed + i) for i in range(3)]
    x = gen.make_input(71 + seed, batch, m.in_c, m.in_h, m.in_w, "normal", "bf16")
    g = harness.GpuDag([(m, blobs[0], None), (m, blobs[1], None), (m, blobs[2], "f32")], batch)
    try:
        names = sorted({L.name.decode() for L in g.dag.launches()})
        ys = g.run(x)
    finally:
        g.close()
    print(f"seed {seed}: input {m.in_c}x{m.in_h}x{m.in_w}, {len(m.layers)} nodes, {m.macs() / 1e9:.2f} GMAC/image, kernels {names}", flush=True)
    refs = harness.oracle_units([(m, blobs[0], x, False), (m, blobs[0], x, True), (m, blobs[1], x, False), (m, blobs[1], x, True), (m, blobs[2], x, False)])
    L = m.layers[m.output]

    def nhwc(r):
        return r.reshape(batch, L.cout, L.out_h, L.out_w).transpose(0, 2, 3, 1).reshape(batch, -1)
    for i in range(2):
        ref_f, ref_s = nhwc(refs[2 * i]), nhwc(refs[2 * i + 1])
        assert ys[i].shape == ref_f.shape and np.isfinite(ys[i]).all()
        floor = 1e-5 * np.sqrt(ref_f.size) / max(float(np.linalg.norm(ref_f)), 1e-30)
        d_sf = harness.rel_l2(ref_s, ref_f)
        assert harness.rel_l2(ys[i], ref_s) <= max(2e-3, 0.5 * d_sf) + floor, (i, harness.rel_l2(ys[i], ref_s), d_sf)
        if d_sf <= 0.5 * BF16_TOL:
            assert harness.rel_l2(ys[i], ref_f) <= BF16_TOL + floor
    ref_w = nhwc(refs[4])
    floor = 1e-5 * np.sqrt(ref_w.size) / max(float(np.linalg.norm(ref_w)), 1e-30)
    assert harness.rel_l2(ys[2], ref_w) <= WIDE_TOL + floor


@pytest.mark.parametrize("seed", range(0, 72, 3))
def test_random_graphs_with_concatenating_blocks(seed):
    """Random graphs in which dense layers, modules with a pooling branch and slice / branch / concatenate units sit
    between the random operators (channel counts in multiples of 8): concatenations written in place next to ones
    that must copy, affine nodes absorbed by their convolution next to ones with other readers.  Two members; the
    optimised schedule equals, bit for bit, the schedule that copies every concatenation and launches every affine
    node, and that plain schedule's bf16 member meets the oracle as in the test above."""
    from tests import harness
    first = randnet.random_model(seed, aligned=True)
    second = randnet.random_model(seed + 1000, in_c=first.in_c, hw=(first.in_h, first.in_w), aligned=True)
    batch = 1 + seed % 3
    mem = [(m, gen.make_blob(m, 8000 + seed + i), None) for i, m in enumerate((first, second))]
    x = gen.make_input(77 + seed, batch, first.in_c, first.in_h, first.in_w, "normal", "bf16")
    print(f"seed {seed}: batch {batch}, input {first.in_c}x{first.in_h}x{first.in_w}, nodes {[len(m[0].layers) for m in mem]}", flush=True)
    res, launches = {}, {}
    for key, kw in (("fast", {}), ("plain", dict(copy_concats=True, separate_affine=True)), ("graph", dict(use_graph=True)),
                    ("ungrouped", dict(group_levels=False)), ("serial", dict(serial_lanes=True))):
        g = harness.GpuDag(mem, batch + 1, **kw)
        try:
            launches[key] = g.dag.query().n_launches
            res[key] = g.run(x)
        finally:
            g.close()
    assert launches["fast"] <= launches["plain"]
    for key in ("plain", "graph", "ungrouped", "serial"):   # (the folded schedule also replayed as a HIP graph, ungrouped, on one stream)
        for i, (y0, y1) in enumerate(zip(res["fast"], res[key])):
            assert np.array_equal(y0, y1, equal_nan=True), f"member {i}: the folded schedule differs from {key}"
    for i, (m, blob, _) in enumerate(mem):
        y = res["fast"][i]
        ref_f = harness.oracle_nhwc(m, blob, x, False)
        ref_s = harness.oracle_nhwc(m, blob, x, True)
        if not (np.isfinite(ref_f).all() and np.isfinite(ref_s).all()):
            continue   # a graph whose activations overflow with these weights has no parity target
        assert y.shape == ref_f.shape and np.isfinite(y).all()
        scale = max(float(np.linalg.norm(ref_f)), 1e-30)
        floor = 1e-5 * np.sqrt(ref_f.size) / scale
        d_sf = harness.rel_l2(ref_s, ref_f)
        e_s = harness.rel_l2(y, ref_s)
        assert e_s <= max(2e-3, 0.5 * d_sf) + floor, f"member {i}: rel L2 vs storage-rounding oracle {e_s}, modes differ by {d_sf}"
