"""CPU-only tests of the library's host side: the C-ABI loads and exports every declared
symbol, DAG compilation (union, levels, grouping), the weight-arena and activation-arena
planners, packing, the state machine and the error paths.  No kernel is launched."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2410_21120_amd as fi
from workloads import gen, zoo

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _build(fams, batch, hw=64, group=True, act=None, seed0=1000, **kw):
    alloc = fi.HostAllocators()
    specs, keep, models = [], [], []
    for i, f in enumerate(fams):
        m = zoo.tiny_cnn() if f == "tiny" else zoo.FAMILIES[f](hw=hw)
        blob = gen.make_blob(m, seed0 + i)
        s, k = fi.make_spec(m, blob.ctypes.data, blob.nbytes, act_dtype=act)
        specs.append(s)
        keep.append((k, blob))
        models.append(m)
    return fi.Dag(specs, batch, alloc, group_levels=group, keepalive=keep, **kw), models, alloc


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "fusedinf.h")).read()
    declared = set(re.findall(r"\b(fi_[a-z_0-9]+)\s*\(", header))
    declared -= {"fi_dag"}
    assert declared == set(fi.EXPORTS)
    lib = C.CDLL(fi.LIB_PATH)
    for name in declared:
        assert getattr(lib, name) is not None
    assert fi.fi_version().startswith("fusedinf")


def test_union_levels_and_operator_count():
    """The DAG is the disjoint union of the members: node count = sum of node counts, per-member
    levels equal the member's own depth (Algorithm 1, compilation loop; Section IV-C: the DAG holds
    exactly the members' operators)."""
    fams = ["resnet50", "mobilenetv2", "vgg16", "resnet18"]
    d, models, _ = _build(fams, 2, separate_chains=True, separate_stem=True)   # one launch per node and level (chained and stem launches: tested below)
    q = d.query()
    assert q.n_models == 4 and q.n_nodes == sum(len(m.layers) for m in models)
    assert q.n_levels == max(max(m.levels()) for m in models)
    assert q.macs_per_image == sum(m.macs() for m in models)
    nodes = d.nodes()
    k = 0
    for mi, m in enumerate(models):
        lv = m.levels()
        for i, L in enumerate(m.layers):
            n = nodes[k]
            assert (n.model, n.index, n.level) == (mi, i, lv[i])
            assert (n.out_c, n.out_h, n.out_w) == (L.cout, L.out_h, L.out_w)
            assert n.is_output == (i == m.output)
            k += 1
    # every launch is homogeneous in level and holds at most FI_MAX_GROUP problems from distinct nodes
    launches = d.launches()
    seen = set()
    for li, L in enumerate(launches):
        assert 1 <= L.n_problems <= fi.FI_MAX_GROUP
        members = [n for n in nodes if n.launch == li and not (L.level == 0)]
        if L.level > 0 and L.name != b"splitk_reduce":  # the reduce launch re-visits its FC launch's nodes
            assert len(members) == L.n_problems and all(n.level == L.level for n in members)
            for n in members:
                assert (n.model, n.index) not in seen
                seen.add((n.model, n.index))
    assert len(seen) == q.n_nodes
    assert [L.level for L in launches] == sorted(L.level for L in launches)


def test_grouping_reduces_launches_only():
    fams = ["resnet50"] * 8
    g, _, _ = _build(fams, 4, separate_chains=True, separate_stem=True)
    u, _, _ = _build(fams, 4, group=False, separate_chains=True, separate_stem=True)   # (a launch per node: chains would take three nodes each, a stem launch two)
    qg, qu = g.query(), u.query()
    n_red = sum(1 for L in u.launches() if L.name == b"splitk_reduce")  # split-K launches have a reduce twin
    assert n_red >= sum(1 for n in u.nodes() if n.op == fi.FI_FC)
    assert qu.n_launches == 1 + qu.n_nodes + n_red
    assert qg.n_launches <= 2 * (1 + qg.n_levels) + 8 and qg.n_nodes == qu.n_nodes
    assert qg.arena_bytes == qu.arena_bytes + (0)  # same weights either way (tables are per node)
    assert qg.act_bytes == qu.act_bytes


def test_activation_arena_liveness_non_overlap():
    for fams in (["resnet50", "mobilenetv2", "vgg16"], ["resnet18"] * 3, ["tiny", "tiny"]):
        d, _, _ = _build(fams, 3, hw=64 if fams[0] != "tiny" else 32)
        q = d.query()
        nodes = [n for n in d.nodes() if n.out_bytes]
        for n in nodes:
            assert n.out_off % 256 == 0 and n.out_off + n.out_bytes <= q.act_bytes
            assert n.first_level <= n.level and n.last_level >= n.first_level   # (a chain's outputs are written at its head's place)
        for i, a in enumerate(nodes):
            for b in nodes[i + 1:]:
                if a.first_level <= b.last_level and b.first_level <= a.last_level:  # alive together
                    assert a.out_off + a.out_bytes <= b.out_off or b.out_off + b.out_bytes <= a.out_off
        # reuse happens: the arena is smaller than the sum of all tensors
        assert q.act_bytes < sum(n.out_bytes for n in nodes) or len(nodes) < 8


def test_consumers_extend_live_ranges():
    d, models, _ = _build(["resnet18"], 1)
    nodes = d.nodes()
    m = models[0]
    for i, L in enumerate(m.layers):
        for src in (L.input, L.residual):
            if src >= 0:
                assert nodes[src].last_level >= nodes[i].level


def test_weight_arena_layout_and_one_copy_accounting():
    d, models, alloc = _build(["resnet18", "vgg16"], 1, hw=32)
    q = d.query()
    assert q.n_device_allocs == 1 and q.n_h2d_copies == 1 and alloc.n_pin == 1
    assert q.device_bytes == q.arena_bytes + q.act_bytes + q.workspace_bytes
    spans = sorted((n.w_off, n.b_off) for n in d.nodes() if n.op in (fi.FI_CONV2D, fi.FI_FC, fi.FI_DWCONV2D))
    flat = [v for s in spans for v in s]
    assert flat == sorted(flat) and all(v % 256 == 0 and v < q.arena_bytes for v in flat)
    d2, _, _ = _build(["resnet18", "vgg16"], 1, hw=32)
    assert d2.query().arena_bytes == q.arena_bytes  # deterministic


def test_pack_is_a_permutation_with_zero_padding():
    m = zoo.mobilenetv2(hw=32)
    blob = gen.make_blob(m, 5)
    spec, keep = fi.make_spec(m, blob.ctypes.data, blob.nbytes)
    n = fi.fi_model_packed_size(spec)
    dst = np.full(n, 0xAB, np.uint8)
    fi.fi_model_pack(spec, dst.ctypes.data, n)
    pk = dst.view(np.uint16)
    # first conv: 3 -> 32, k3, reading the 4-channel staged input: packed rows [o][r][s][c padded to 4],
    # row length 36 -> 64
    L = m.layers[0]
    w = blob[L.w_off:L.w_off + 2 * 32 * 27].view(np.uint16).reshape(32, 3, 3, 3)
    rows = pk[:32 * 64].reshape(32, 64)
    assert np.array_equal(rows[:, :36].reshape(32, 3, 3, 4)[..., :3], w.transpose(0, 2, 3, 1))
    assert not rows[:, :36].reshape(32, 3, 3, 4)[..., 3:].any() and not rows[:, 36:].any()
    # second conv (1x1, 32 -> 16 after the depthwise): channels are padded to 8 everywhere else
    L2 = m.layers[2]
    assert L2.op == "conv" and L2.cin == 32
    # multiset of non-zero weights is preserved over the whole blob
    canon = np.concatenate([blob[L.w_off:L.w_off + 2 * (L.cout * (L.cin if L.op != "dwconv" else 1) * L.k * L.k)].view(np.uint16)
                            for L in m.layers if L.op in ("conv", "dwconv", "fc")])
    with pytest.raises(fi.FiError):
        fi.fi_model_pack(spec, dst.ctypes.data, n - 1)
    assert n % 256 == 0 and n >= canon.nbytes


def test_fc_weights_are_packed_in_matrix_core_blocks():
    """bf16 FC weights: rows over (h, w, c padded to 8), cut into blocks of 32 features x 16 reduction elements
    stored in the order the 64 lanes of a wave load them (lane l: feature l % 32, elements (l / 32) * 8 .. + 8),
    so one block is one contiguous kilobyte; features past cout are zero rows."""
    m = zoo.Model("f", "bf16", 5, 2, 3)
    m.add(zoo.FC, -1, cin=30, cout=40)
    m.shapes()
    blob = gen.make_blob(m, 9)
    spec, keep = fi.make_spec(m, blob.ctypes.data, blob.nbytes)
    n = fi.fi_model_packed_size(spec)
    dst = np.full(n, 0xAB, np.uint8)
    fi.fi_model_pack(spec, dst.ctypes.data, n)
    L = m.layers[0]
    w = blob[L.w_off:L.w_off + 2 * 40 * 30].view(np.uint16).reshape(40, 5, 2, 3)
    kp = 64                                    # 2 * 3 pixels x 8 padded channels = 48, rounded up to 32s
    rows = np.zeros((64, kp), np.uint16)       # 40 features padded to two tiles of 32
    rows[:40, :48].reshape(40, 2, 3, 8)[..., :5] = w.transpose(0, 2, 3, 1)
    steps = kp // 16
    blocks = dst[:2 * 64 * kp].view(np.uint16).reshape(2, steps, 64, 8)
    for t in range(2):
        for s_ in range(steps):
            for lane in range(64):
                f, k0 = t * 32 + lane % 32, s_ * 16 + (lane // 32) * 8
                assert np.array_equal(blocks[t, s_, lane], rows[f, k0:k0 + 8]), (t, s_, lane)


def test_packed_and_canonical_members_build_the_same_image():
    m = zoo.resnet18(hw=32)
    blob = gen.make_blob(m, 9)
    spec, keep = fi.make_spec(m, blob.ctypes.data, blob.nbytes)
    n = fi.fi_model_packed_size(spec)
    packed = np.zeros(n, np.uint8)
    fi.fi_model_pack(spec, packed.ctypes.data, n)
    a1, a2 = fi.HostAllocators(), fi.HostAllocators()
    d1 = fi.Dag([spec], 1, a1, keepalive=keep)
    spec2, keep2 = fi.make_spec(m, packed.ctypes.data, n, packed=True)
    d2 = fi.Dag([spec2], 1, a2, keepalive=keep2)
    i1 = bytes(next(iter(a1.live.values())))[:d1.query().arena_bytes]
    i2 = bytes(next(iter(a2.live.values())))[:d2.query().arena_bytes]
    assert i1 == i2


def _spec_with(mutator, fam="tiny"):
    m = zoo.tiny_cnn() if fam == "tiny" else zoo.FAMILIES[fam](hw=32)
    blob = gen.make_blob(m, 1)
    spec, keep = fi.make_spec(m, blob.ctypes.data, blob.nbytes)
    mutator(spec)
    return spec, (keep, blob)


@pytest.mark.parametrize("mutate,status", [
    (lambda s: setattr(s.layers[2], "input", 3), fi.FI_EINVAL),           # edge to a later node (cycle)
    (lambda s: setattr(s.layers[2], "input", 77), fi.FI_EINVAL),          # dangling edge
    (lambda s: setattr(s.layers[2], "cin", 17), fi.FI_EINVAL),            # shape mismatch
    (lambda s: setattr(s.layers[0], "op", 42), fi.FI_EUNSUPPORTED),       # unknown operator
    (lambda s: setattr(s.layers[1], "kw", 3), fi.FI_EUNSUPPORTED),        # non-square pooling window
    (lambda s: setattr(s.layers[0], "kw", 16), fi.FI_EUNSUPPORTED),       # kernel wider than 15
    (lambda s: setattr(s.layers[2], "residual", 0), fi.FI_EINVAL),        # residual shape mismatch
    (lambda s: setattr(s.layers[4], "w_off", 1 << 40), fi.FI_EINVAL),     # weights past the blob
    (lambda s: setattr(s, "output_node", 99), fi.FI_EINVAL),
    (lambda s: setattr(s, "act_dtype", fi.FI_BF16), fi.FI_EINVAL),        # fp32 weights need fp32 activations
    (lambda s: setattr(s, "n_layers", 0), fi.FI_EINVAL),
])
def test_malformed_specs_are_refused(mutate, status):
    spec, keep = _spec_with(mutate)
    alloc = fi.HostAllocators()
    with pytest.raises(fi.FiError) as e:
        fi.Dag([spec], 1, alloc, keepalive=keep)
    assert e.value.status == status and fi.fi_last_error()
    assert alloc.n_pin == 0 or not alloc.live  # nothing leaked


def test_members_must_share_dtype_and_input_shape():
    a, ka = _spec_with(lambda s: None)
    b, kb = _spec_with(lambda s: None, fam="resnet18")
    with pytest.raises(fi.FiError) as e:
        fi.Dag([a, b], 1, fi.HostAllocators(), keepalive=(ka, kb))
    assert e.value.status == fi.FI_EINVAL


def test_budget_state_machine_and_device_oom():
    d, _, alloc = _build(["resnet18"], 1, hw=32)
    need = d.query().device_bytes
    with pytest.raises(fi.FiError) as e:
        _build(["resnet18"], 1, hw=32, max_device_bytes=need - 1)
    assert e.value.status == fi.FI_EBUDGET
    _build(["resnet18"], 1, hw=32, max_device_bytes=need)[0].destroy()
    # not loaded: run / unload are state errors
    outs = (C.c_void_p * 1)(1)
    assert fi.lib().fi_run(d.h, C.c_void_p(1), 1, outs, None) == fi.FI_ESTATE
    assert fi.lib().fi_unload(d.h) == fi.FI_ESTATE
    # the device allocator refuses: FI_ENOMEM_DEVICE, handle stays BUILT and can be destroyed
    with pytest.raises(fi.FiError) as e:
        d.load()
    assert e.value.status == fi.FI_ENOMEM_DEVICE and alloc.n_dev == 1 and d.query().state == 0
    d.destroy()
    assert not alloc.live  # pinned image returned
    # argument checks
    assert fi.lib().fi_query(None, None) == fi.FI_EINVAL
    bad = fi.fi_build_opts()
    bad.max_batch = 0
    h = C.c_void_p()
    s, k = _spec_with(lambda s: None)
    assert fi.lib().fi_build_dag(C.byref(s), 1, C.byref(bad), C.byref(h)) == fi.FI_EINVAL and not h.value
    fi.fi_destroy(None)


def test_per_model_load_mode_needs_packed_members():
    with pytest.raises(fi.FiError) as e:
        _build(["resnet18"], 1, hw=32, load_mode=fi.FI_LOAD_PER_MODEL)
    assert e.value.status == fi.FI_EINVAL


def test_lanes_group_members_of_identical_architecture():
    """Members with identical graphs share a lane (and their launches); different architectures get their
    own lane, whose tensors and split-K scratch never share memory with another lane's."""
    d, _, _ = _build(["resnet18", "vgg16", "resnet18", "mobilenetv2"], 2)
    q = d.query()
    assert q.n_lanes == 3
    nodes, launches = d.nodes(), d.launches()
    lane_of_model = {}
    for n in nodes:
        lane_of_model.setdefault(n.model, launches[n.launch].lane)
        assert launches[n.launch].lane == lane_of_model[n.model]
    assert lane_of_model[0] == lane_of_model[2] and len({lane_of_model[m] for m in (0, 1, 3)}) == 3
    stored = [n for n in nodes if n.out_bytes]
    for i, a in enumerate(stored):
        for b in stored[i + 1:]:
            if lane_of_model[a.model] != lane_of_model[b.model]:
                assert a.out_off + a.out_bytes <= b.out_off or b.out_off + b.out_bytes <= a.out_off
    one, _, _ = _build(["resnet18"] * 3, 2)
    assert one.query().n_lanes == 1
    ser, _, _ = _build(["resnet18", "vgg16"], 2, serial_lanes=True)
    assert ser.query().n_lanes == 1


def test_large_family_is_halved_into_two_lanes():
    """Four or more identical members whose convolutions cover the chip even at half the family run as
    two lanes (first half, second half); the same family at a small batch stays one lane."""
    big, _, _ = _build(["resnet18"] * 4, 256)
    assert big.query().n_lanes == 2
    launches = big.launches()
    lane_of_model = {}
    for n in big.nodes():
        lane_of_model.setdefault(n.model, launches[n.launch].lane)
        assert launches[n.launch].lane == lane_of_model[n.model]
    assert [lane_of_model[m] for m in range(4)] == [0, 0, 1, 1]
    small, _, _ = _build(["resnet18"] * 4, 2)
    assert small.query().n_lanes == 1
    ser, _, _ = _build(["resnet18"] * 4, 256, serial_lanes=True)
    assert ser.query().n_lanes == 1


def test_swap_model_replans_without_moving_the_other_members():
    """Individual model swap (Section V, Table IV): the other members keep their arena offsets, the
    newcomer takes the lowest gap that holds it, and the schedule is that of a fresh build of the
    new member set (same nodes, levels and launch count)."""
    d, models, _ = _build(["resnet18", "vgg16", "mobilenetv2"], 2)
    before = d.members()
    m_new = zoo.FAMILIES["resnet18"](hw=64)
    blob = gen.make_blob(m_new, 77)
    spec, keep = fi.make_spec(m_new, blob.ctypes.data, blob.nbytes)
    d.swap_model(1, spec, keepalive=(keep, blob))      # vgg16 (large) -> resnet18 (smaller): fits the gap
    after = d.members()
    assert (after[0].arena_off, after[2].arena_off) == (before[0].arena_off, before[2].arena_off)
    assert after[1].arena_off == before[1].arena_off and after[1].packed_bytes < before[1].packed_bytes
    fresh, _, _ = _build(["resnet18", "resnet18", "mobilenetv2"], 2)
    qa, qb = d.query(), fresh.query()
    assert (qa.n_nodes, qa.n_levels, qa.n_launches, qa.n_lanes, qa.act_bytes, qa.macs_per_image) == \
           (qb.n_nodes, qb.n_levels, qb.n_launches, qb.n_lanes, qb.act_bytes, qb.macs_per_image)
    assert qa.arena_bytes >= qb.arena_bytes          # the gap the larger member left is still inside the arena
    for na, nb in zip(d.nodes(), fresh.nodes()):
        assert (na.model, na.index, na.op, na.level, na.out_off) == (nb.model, nb.index, nb.op, nb.level, nb.out_off)
    # a larger newcomer does not fit the gap: it goes past the last member and the arena grows
    big = zoo.FAMILIES["vgg16"](hw=64)
    bblob = gen.make_blob(big, 78)
    bspec, bkeep = fi.make_spec(big, bblob.ctypes.data, bblob.nbytes)
    d.swap_model(0, bspec, keepalive=(bkeep, bblob))
    again = d.members()
    assert again[1].arena_off == after[1].arena_off and again[2].arena_off == after[2].arena_off
    spans = sorted((m.arena_off, m.arena_off + m.packed_bytes) for m in again)
    assert all(a[1] <= b[0] for a, b in zip(spans, spans[1:]))
    assert d.query().arena_bytes >= spans[-1][1]


def test_shrinking_swap_on_a_built_handle_shrinks_the_arena_the_next_load_copies():
    """The last-placed large member gives way to a small one: the plan's weight arena (what a one-copy load
    moves) shrinks to the members that are left, and the device footprint with it."""
    d, _, _ = _build(["resnet18", "vgg16"], 2)
    q0 = d.query()
    m_new = zoo.FAMILIES["mobilenetv2"](hw=64)
    blob = gen.make_blob(m_new, 79)
    spec, keep = fi.make_spec(m_new, blob.ctypes.data, blob.nbytes)
    d.swap_model(1, spec, keepalive=(keep, blob))
    q1 = d.query()
    spans = sorted((m.arena_off, m.arena_off + m.packed_bytes) for m in d.members())
    assert q1.arena_bytes < q0.arena_bytes // 2
    assert spans[-1][1] <= q1.arena_bytes < spans[-1][1] + 256
    assert q1.device_bytes == q1.arena_bytes + q1.act_bytes + q1.workspace_bytes < q0.device_bytes
    fresh, _, _ = _build(["resnet18", "mobilenetv2"], 2)
    assert fresh.query().arena_bytes == q1.arena_bytes


def test_swap_model_errors_leave_the_dag_unchanged():
    d, _, _ = _build(["resnet18", "resnet18"], 2)
    q0 = d.query()
    off0 = [(m.arena_off, m.packed_bytes) for m in d.members()]
    other = zoo.FAMILIES["resnet18"](hw=32)            # different input shape
    blob = gen.make_blob(other, 5)
    spec, keep = fi.make_spec(other, blob.ctypes.data, blob.nbytes)
    with pytest.raises(fi.FiError) as e:
        d.swap_model(0, spec, keepalive=(keep, blob))
    assert e.value.status == fi.FI_EINVAL
    ok = zoo.FAMILIES["resnet18"](hw=64)
    okb = gen.make_blob(ok, 6)
    okspec, okkeep = fi.make_spec(ok, okb.ctypes.data, okb.nbytes)
    for bad_slot in (-1, 2):
        with pytest.raises(fi.FiError) as e:
            d.swap_model(bad_slot, okspec, keepalive=(okkeep, okb))
        assert e.value.status == fi.FI_EINVAL
    q1 = d.query()
    assert (q1.n_nodes, q1.n_launches, q1.arena_bytes, q1.act_bytes) == (q0.n_nodes, q0.n_launches, q0.arena_bytes, q0.act_bytes)
    assert [(m.arena_off, m.packed_bytes) for m in d.members()] == off0
    # a budget that the larger member set would exceed: FI_EBUDGET, nothing changes
    tight, _, _ = _build(["resnet18", "resnet18"], 2, max_device_bytes=q0.device_bytes + 4096)
    big = zoo.FAMILIES["vgg16"](hw=64)
    bb = gen.make_blob(big, 9)
    bspec, bkeep = fi.make_spec(big, bb.ctypes.data, bb.nbytes)
    with pytest.raises(fi.FiError) as e:
        tight.swap_model(1, bspec, keepalive=(bkeep, bb))
    assert e.value.status == fi.FI_EBUDGET
    assert tight.query().n_nodes == q0.n_nodes


def _specs(fams, hw=64, seed0=1000):
    specs, keep = [], []
    for i, f in enumerate(fams):
        m = zoo.FAMILIES[f](hw=hw)
        blob = gen.make_blob(m, seed0 + i)
        sp, k = fi.make_spec(m, blob.ctypes.data, blob.nbytes)
        specs.append(sp)
        keep.append((k, blob))
    return specs, keep


def test_footprint_equals_the_built_dag_without_touching_weights():
    fams = ["resnet18", "mobilenetv2", "resnet18"]
    specs, keep = _specs(fams)
    alloc = fi.HostAllocators()
    opts = fi.make_opts(4, alloc)
    fp = fi.fi_footprint(specs, opts)
    d = fi.Dag(specs, 4, alloc, keepalive=keep)
    q = d.query()
    assert (fp.arena_bytes, fp.act_bytes, fp.workspace_bytes, fp.device_bytes, fp.n_nodes, fp.n_launches, fp.n_lanes) == \
           (q.arena_bytes, q.act_bytes, q.workspace_bytes, q.device_bytes, q.n_nodes, q.n_launches, q.n_lanes)
    # the footprint needs the architecture only: a spec whose weight pointer leads nowhere readable still answers
    ghost = []
    for sp in specs:
        g = fi.fi_model_spec.from_buffer_copy(sp)
        g.weights = 4096
        ghost.append(g)
    assert fi.fi_footprint(ghost, opts).device_bytes == q.device_bytes


def test_partition_first_fit_in_order_within_budget():
    """Manager batching (Section IV): batches in the caller's order, each within the budget by the exact
    footprint of its DAG; a budget below one model's need is refused."""
    fams = ["resnet18", "vgg16", "mobilenetv2", "resnet50", "resnet18", "vgg16", "mobilenetv2"]
    specs, keep = _specs(fams)
    opts = fi.make_opts(4, fi.HostAllocators())
    single = [fi.fi_footprint([sp], opts).device_bytes for sp in specs]
    everything = fi.fi_footprint(specs, opts).device_bytes
    group_of, n = fi.fi_partition(specs, opts, everything)
    assert n == 1 and group_of == [0] * len(fams)
    budget = max(single) + min(single)                  # room for the largest model plus a small one
    group_of, n = fi.fi_partition(specs, opts, budget)
    assert n > 1 and group_of == sorted(group_of) and group_of[0] == 0 and group_of[-1] == n - 1
    for g in range(n):
        members = [sp for sp, go in zip(specs, group_of) if go == g]
        assert fi.fi_footprint(members, opts).device_bytes <= budget
        nxt = [sp for sp, go in zip(specs, group_of) if go == g + 1][:1]
        if nxt:                                         # first fit: the next model would not have fitted
            assert fi.fi_footprint(members + nxt, opts).device_bytes > budget
    with pytest.raises(fi.FiError) as e:
        fi.fi_partition(specs, opts, max(single) - 1)
    assert e.value.status == fi.FI_EBUDGET


def test_per_member_inputs_stage_one_copy_per_member():
    """With per-member inputs (Algorithm 1's x^m) the staging level holds one problem per member and the
    activation arena one staged copy per member; the rest of the schedule is unchanged."""
    fams = ["resnet18", "resnet18", "mobilenetv2"]
    shared, _, _ = _build(fams, 2)
    own, _, _ = _build(fams, 2, per_member_inputs=True)
    ls, lo = shared.launches(), own.launches()
    assert [L.n_problems for L in ls if L.level == 0] == [1]
    assert sum(L.n_problems for L in lo if L.level == 0) == len(fams)
    assert [(L.level, L.name, L.n_problems) for L in ls if L.level > 0] == [(L.level, L.name, L.n_problems) for L in lo if L.level > 0]
    qs, qo = shared.query(), own.query()
    assert (qo.n_nodes, qo.n_levels, qo.arena_bytes) == (qs.n_nodes, qs.n_levels, qs.arena_bytes)


def test_maximum_sizes_are_refused_at_build_time():
    """The MFMA convolution addresses its input through a 32-bit buffer resource and decodes output rows
    with exact float arithmetic: more than 2^24 output pixels per launch, or an input tensor of 2 GiB or
    more, is refused when the DAG is built, never at run time."""
    alloc = fi.HostAllocators()
    m = zoo.Model("wide_input", "bf16", 1024, 32, 32)   # one image = 32 x 32 x 1024 bf16 = 2 MiB
    m.add(zoo.CONV, -1, cin=1024, cout=8, k=1, stride=1, pad=0, act=zoo.RELU)
    m.shapes()
    blob = gen.make_blob(m, 1)
    spec, keep = fi.make_spec(m, blob.ctypes.data, blob.nbytes)
    assert fi.fi_footprint([spec], fi.make_opts(1023, alloc)).device_bytes > 0
    with pytest.raises(fi.FiError) as e:
        fi.fi_footprint([spec], fi.make_opts(1024, alloc))   # 1024 x 2 MiB = 2^31
    assert e.value.status == fi.FI_EUNSUPPORTED and "2 GiB" in str(e.value)
    r = zoo.FAMILIES["resnet18"](hw=64)                 # stem output 32 x 32 pixels per image
    rb = gen.make_blob(r, 2)
    rspec, rkeep = fi.make_spec(r, rb.ctypes.data, rb.nbytes)
    assert fi.fi_footprint([rspec], fi.make_opts((1 << 14) - 1, alloc)).n_nodes == len(r.layers)
    with pytest.raises(fi.FiError) as e:
        fi.fi_footprint([rspec], fi.make_opts(1 << 14, alloc))   # 2^14 x 2^10 = 2^24 output pixels
    assert e.value.status == fi.FI_EUNSUPPORTED and "2^24" in str(e.value)


def test_concat_and_ceil_pooling_in_the_planner():
    """A concat node has the channels of both sources and reads both (live ranges extend to it); pooling with
    ceil_mode takes the rounded-up size; malformed concats are refused."""
    m = zoo.Model("cat", "bf16", 8, 9, 9)
    a = m.add(zoo.CONV, -1, cin=8, cout=16, k=1, stride=1, pad=0, act=zoo.RELU)
    b = m.add(zoo.CONV, -1, cin=8, cout=24, k=3, stride=1, pad=1, act=zoo.RELU)
    c = m.add(zoo.CONCAT, a, residual=b)
    p = m.add(zoo.MAXPOOL, c, k=2, stride=2, pad=0, ceil=True)
    m.add(zoo.CONV, p, cin=40, cout=10, k=1, stride=1, pad=0)
    m.shapes()
    blob = gen.make_blob(m, 1)
    spec, keep = fi.make_spec(m, blob.ctypes.data, blob.nbytes)
    d = fi.Dag([spec], 2, fi.HostAllocators(), keepalive=keep)
    nodes = d.nodes()
    assert (nodes[2].out_c, nodes[2].out_h, nodes[2].out_w) == (40, 9, 9)
    assert (nodes[3].out_h, nodes[3].out_w) == (5, 5)                      # floor would give 4
    assert nodes[0].last_level >= nodes[2].level and nodes[1].last_level >= nodes[2].level
    # both sources are convolutions nobody else reads: they are written straight into the concatenation's tensor
    # (16 channels of the first, then the second), which lives from the first of them on and needs no launch
    assert "concat" not in [L.name.decode() for L in d.launches()]
    # the handle tells its caller how large the buffers of a run are
    assert d.query().input_image_bytes == 9 * 9 * 8 * 2 and d.members()[0].output_row_bytes == 5 * 5 * 10 * 4
    assert nodes[0].out_bytes == 0 and nodes[1].out_bytes == 0 and nodes[2].out_bytes >= 2 * 9 * 9 * 40 * 2
    assert nodes[0].out_off == nodes[2].out_off and nodes[1].out_off == nodes[2].out_off + 16 * 2
    assert nodes[2].first_level <= min(nodes[0].level, nodes[1].level)
    assert nodes[2].launch == nodes[1].launch
    # ... unless the handle is built to copy
    spec_c, keep_c = fi.make_spec(m, blob.ctypes.data, blob.nbytes)
    dc = fi.Dag([spec_c], 2, fi.HostAllocators(), keepalive=keep_c, copy_concats=True)
    assert "concat" in [L.name.decode() for L in dc.launches()]
    assert all(n.out_bytes > 0 for n in dc.nodes()[:3])
    assert dc.query().n_launches == d.query().n_launches + 1

    def broken(edit):
        spec2, keep2 = fi.make_spec(m, blob.ctypes.data, blob.nbytes)
        edit(spec2)
        with pytest.raises(fi.FiError) as e:
            fi.Dag([spec2], 2, fi.HostAllocators(), keepalive=keep2)
        return e.value.status
    assert broken(lambda s: setattr(s.layers[2], "residual", fi.FI_NO_RESIDUAL)) == fi.FI_EINVAL     # no second source
    assert broken(lambda s: setattr(s.layers[2], "cout", 41)) == fi.FI_EINVAL                        # wrong channel sum
    assert broken(lambda s: setattr(s.layers[2], "act", fi.FI_ACT_RELU)) == fi.FI_EUNSUPPORTED
    assert broken(lambda s: setattr(s.layers[1], "stride", 2)) == fi.FI_EINVAL                       # sources differ in size


@pytest.mark.parametrize("seed", range(0, 60, 3))
def test_random_graphs_compile_into_one_dag(seed):
    """Three random layer graphs over every operator, sharing the input shape, compile into one DAG that holds
    exactly their nodes, with every tensor inside the planned arenas."""
    from workloads import randnet
    first = randnet.random_model(seed)
    models = [first] + [randnet.random_model(seed + j, in_c=first.in_c, hw=(first.in_h, first.in_w)) for j in (1, 2)]
    alloc = fi.HostAllocators()
    specs, keep = [], []
    for i, m in enumerate(models):
        blob = gen.make_blob(m, 7000 + seed + i)
        s, k = fi.make_spec(m, blob.ctypes.data, blob.nbytes, act_dtype="f32" if i == 2 else None)
        specs.append(s)
        keep.append((k, blob))
    d = fi.Dag(specs, 3, alloc, keepalive=keep)
    q = d.query()
    assert q.n_nodes == sum(len(m.layers) for m in models) and q.n_models == 3
    assert q.macs_per_image == sum(m.macs() for m in models)
    nodes = d.nodes()
    k = 0
    for m in models:
        for L in m.layers:
            n = nodes[k]
            assert (n.out_c, n.out_h, n.out_w) == (L.cout, L.out_h, L.out_w)
            assert n.is_output or n.out_off + n.out_bytes <= q.act_bytes
            k += 1
    d.destroy()


def test_server_refuses_an_unloaded_dag():
    """The request aggregator needs a LOADED DAG built for per-member inputs; the check comes before any device call."""
    d, _, _ = _build(["resnet18"], 2, hw=32, per_member_inputs=True)
    with pytest.raises(fi.FiError) as e:
        fi.Server(d)
    assert e.value.status == fi.FI_ESTATE and "not loaded" in str(e.value)
    h = C.c_void_p()
    assert fi.lib().fi_server_start(None, None, C.byref(h)) == fi.FI_EINVAL
    assert fi.lib().fi_server_stop(None) == fi.FI_EINVAL
    d.destroy()


@pytest.mark.parametrize("seed", range(0, 40, 2))
def test_random_graphs_with_concatenating_blocks_compile_both_ways(seed):
    """Random graphs with dense layers, pooling modules and slice / branch / concatenate units: the schedule that stores
    concatenation sources in place and lets convolutions absorb affine nodes has no more launches than the plain one
    (its arena may be a little larger: a concatenation's tensor lives from its first source on), holds the same nodes,
    and every tensor lies inside the arena."""
    from workloads import randnet
    m = randnet.random_model(seed, aligned=True)
    blob = gen.make_blob(m, 5)
    dags = {}
    for key, kw in (("fast", {}), ("plain", dict(copy_concats=True, separate_affine=True))):
        spec, keep = fi.make_spec(m, blob.ctypes.data, blob.nbytes)
        dags[key] = fi.Dag([spec], 3, fi.HostAllocators(), keepalive=(keep, blob), **kw)
    qf, qp = dags["fast"].query(), dags["plain"].query()
    assert qf.n_nodes == qp.n_nodes == len(m.layers)
    assert qf.n_launches <= qp.n_launches
    for n in dags["fast"].nodes():
        assert n.out_off + n.out_bytes <= qf.act_bytes
        assert 0 <= n.launch < qf.n_launches
    ops = [L.op for L in m.layers]
    if "concat" not in ops and not any(L.op == "dwconv" and L.k == 1 for L in m.layers):
        assert qf.n_launches == qp.n_launches


def test_folded_schedules_of_the_concatenating_and_gated_families():
    """What the planner folds, family by family (launch names of the compiled schedule): DenseNet-121 has neither
    concatenation nor affine (depthwise) launches left except the affine nodes a pooling layer reads; GoogLeNet and
    SqueezeNet have no concatenation launch; MobileNetV3 has no scaling launch, with bf16 and with fp32 activations;
    ShuffleNet V2 x1.0 (58-channel halves) has no concatenation launch because its shuffles interleave.  With the two
    build options set the plain schedule is back."""
    def names(fam, act=None, **kw):
        m = zoo.FAMILIES[fam](hw=64)
        blob = gen.make_blob(m, 3)
        spec, keep = fi.make_spec(m, blob.ctypes.data, blob.nbytes, act_dtype=act)
        d = fi.Dag([spec], 2, fi.HostAllocators(), keepalive=(keep, blob), **kw)
        return [L.name.decode() for L in d.launches()], sum(1 for L in m.layers if L.op == "concat"), m
    plain = dict(copy_concats=True, separate_affine=True)
    n, cats, m = names("densenet121")
    affine = sum(1 for L in m.layers if L.op == "dwconv" and L.k == 1)
    assert cats == 58 and "concat" not in n and n.count("dwconv") <= 1 < affine      # only the final normalisation (read by a pooling node) keeps its launch
    n_plain, _, _ = names("densenet121", **plain)
    assert n_plain.count("concat") == 58 and n_plain.count("dwconv") == affine
    for fam in ("googlenet", "squeezenet1_1", "shufflenet_v2_x1_0", "shufflenet_v2_x0_5"):
        n, cats, _ = names(fam)
        assert cats > 0 and "concat" not in n, fam
        assert names(fam, **plain)[0].count("concat") == cats, fam
    for act in (None, "f32"):
        n, _, m = names("mobilenet_v3_large", act)
        gates = sum(1 for L in m.layers if L.op == "mul")
        assert gates == 8 and "channel_scale" not in n
        assert names("mobilenet_v3_large", act, **plain)[0].count("channel_scale") == gates
    # the grouped 3x3 convolutions of ResNeXt run on 64-column tiles (a tile then walks the channels of its own groups only)
    m = zoo.FAMILIES["resnext50_32x4d"](hw=64)
    blob = gen.make_blob(m, 3)
    spec, keep = fi.make_spec(m, blob.ctypes.data, blob.nbytes)
    d = fi.Dag([spec], 2, fi.HostAllocators(), keepalive=(keep, blob))
    launch_names = [L.name.decode() for L in d.launches()]
    grouped = [i for i, L in enumerate(m.layers) if L.op == "conv" and L.groups > 1]
    assert len(grouped) == 16
    assert all(launch_names[d.nodes()[i].launch] in ("conv_mfma_256x64", "conv_mfma_128x64", "conv_mfma_64x64") for i in grouped)


def test_chains_drop_the_first_tensor_and_two_launches_per_block():
    """A bottleneck's 3x3, its 1x1 expansion and the next block's 1x1 reduction run as one launch: the 3x3's output has
    no buffer, the launch's compulsory bytes are the head's input, the second node's residual and output and the third
    node's output, and the schedule has fewer launches than with separate_chains."""
    d, models, _ = _build(["resnet50"] * 2, 8, hw=128)
    p, _, _ = _build(["resnet50"] * 2, 8, hw=128, separate_chains=True)
    names = [L.name.decode() for L in d.launches()]
    assert names.count("conv_chain3") >= 3 and not any(n.decode().startswith("conv_chain") for n in (L.name for L in p.launches()))
    assert d.query().n_launches < p.query().n_launches
    assert d.query().macs_per_image == p.query().macs_per_image
    nodes, pnodes = d.nodes(), p.nodes()
    for L in d.launches():
        if not L.name.decode().startswith("conv_chain"):
            continue
        head = nodes[L.first_node]
        assert head.out_bytes == 0 and pnodes[L.first_node].out_bytes > 0
        assert L.n_problems == 6   # two members, three nodes each
    chained = sum(L.bytes_per_image for L in d.launches())
    plain = sum(L.bytes_per_image for L in p.launches())
    assert chained < 0.95 * plain   # activation bytes per image of the whole schedule (only the first stage chains at this size)
    assert sum(L.macs_per_image for L in d.launches()) == sum(L.macs_per_image for L in p.launches())


def test_stem_launch_takes_the_pool_and_drops_the_first_tensor():
    """The 7x7 stride-2 first convolution and the 3x3 stride-2 max-pool behind it run as one launch carried by the pool
    node: the convolution's output has no buffer, its work is counted under that launch, the compulsory bytes are the
    input image and the pooled tensor, and the staged input stays alive until that launch."""
    d, models, _ = _build(["resnet50", "resnet18", "vgg11"], 4, hw=96)
    p, _, _ = _build(["resnet50", "resnet18", "vgg11"], 4, hw=96, separate_stem=True)
    names = [L.name.decode() for L in d.launches()]
    pnames = [L.name.decode() for L in p.launches()]
    assert "conv_stem_pool" in names and not any(n.startswith("conv_stem") for n in pnames)
    qd, qp = d.query(), p.query()
    assert (qd.n_nodes, qd.n_levels, qd.macs_per_image, qd.arena_bytes) == (qp.n_nodes, qp.n_levels, qp.macs_per_image, qp.arena_bytes)
    assert qd.n_launches < qp.n_launches
    nodes, pnodes = d.nodes(), p.nodes()
    members = d.members()
    for mi in (0, 1):   # the two ResNets
        conv, pool = nodes[members[mi].first_node], nodes[members[mi].first_node + 1]
        assert conv.out_bytes == 0 and pnodes[members[mi].first_node].out_bytes > 0
        assert conv.launch == pool.launch and names[pool.launch] == "conv_stem_pool"
        assert pool.out_bytes == pnodes[members[mi].first_node + 1].out_bytes
    vgg_first = nodes[members[2].first_node]
    assert names[vgg_first.launch] == "conv_stem" and vgg_first.out_bytes > 0   # a 3x3 stride-1 first layer: the stem kernel, no pool to take
    assert pnames[pnodes[members[2].first_node].launch].startswith("conv_mfma")
    for L in d.launches():
        if L.name.decode() != "conv_stem_pool":
            continue
        pool = nodes[L.first_node]
        conv = nodes[L.first_node - 1]
        assert L.macs_per_image >= conv.macs and L.level == pool.level
        # the input image (3 channels) and the pooled tensor (64 channels), bf16, for every problem of the launch
        assert L.bytes_per_image == L.n_problems * 2 * (96 * 96 * 3 + pool.out_h * pool.out_w * 64)
    assert sum(L.macs_per_image for L in d.launches()) == sum(L.macs_per_image for L in p.launches())
    assert sum(L.bytes_per_image for L in d.launches()) < sum(L.bytes_per_image for L in p.launches())
    # a stem whose reader is not that pool keeps a launch of its own, with the stem kernel
    from workloads import zoo
    m = zoo.Model("stem_only", "bf16", 3, 64, 64)
    a = m.add(zoo.CONV, zoo.MODEL_INPUT, cin=3, cout=64, k=7, stride=2, pad=3, act=zoo.RELU)
    a = m.add(zoo.MAXPOOL, a, k=2, stride=2, pad=0)
    m.add(zoo.CONV, a, cin=64, cout=16, k=1, stride=1, pad=0, act=zoo.NONE)
    m.shapes()
    blob = gen.make_blob(m, 77)
    spec, k = fi.make_spec(m, blob.ctypes.data, blob.nbytes)
    alloc = fi.HostAllocators()
    lone = fi.Dag([spec], 2, alloc, keepalive=[(k, blob)])
    lnames = [L.name.decode() for L in lone.launches()]
    assert "conv_stem" in lnames and "maxpool" in lnames and "conv_stem_pool" not in lnames
    assert lone.nodes()[0].out_bytes > 0


def test_member_chunks_shrink_the_activation_arena():
    """The early levels of a lane's members run chunk after chunk: the chunks' early tensors share memory, launches get
    more numerous, the live ranges (in launch order) of tensors that share bytes never overlap."""
    base, _, _ = _build(["resnet50"] * 4 + ["vgg16"] * 2, 4, hw=128)
    half, _, _ = _build(["resnet50"] * 4 + ["vgg16"] * 2, 4, hw=128, member_chunks=2)
    qb, qh = base.query(), half.query()
    assert qh.act_bytes < 0.9 * qb.act_bytes and qh.n_launches > qb.n_launches
    assert (qh.arena_bytes, qh.n_nodes, qh.n_levels, qh.macs_per_image) == (qb.arena_bytes, qb.n_nodes, qb.n_levels, qb.macs_per_image)
    lane_of = [m.lane for m in half.members()]
    nodes = [n for n in half.nodes() if n.out_bytes]
    for i, a in enumerate(nodes):
        for b in nodes[i + 1:]:
            if lane_of[a.model] != lane_of[b.model] or (a.first_level <= b.last_level and b.first_level <= a.last_level):
                assert a.out_off + a.out_bytes <= b.out_off or b.out_off + b.out_bytes <= a.out_off
    # a single member per lane has nothing to chunk
    one, _, _ = _build(["resnet50", "vgg16"], 4, hw=128, member_chunks=2)
    ref, _, _ = _build(["resnet50", "vgg16"], 4, hw=128)
    assert one.query().act_bytes == ref.query().act_bytes and one.query().n_launches == ref.query().n_launches
