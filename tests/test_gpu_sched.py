"""Round-robin scheduling of DAG batches on the GPU (Section IV, "Manager"; Section V, consecutive
swaps), through the C-ABI: whatever the batching, with or without the overlapped load, every model's
output equals, bit for bit, the output of the model run alone, and the counts of loads and runs are
those of the schedule."""
import numpy as np
import pytest

from workloads import gen, zoo

pytestmark = pytest.mark.gpu

HW = 64
FAMS = [("resnet18", None), ("vgg16", None), ("mobilenetv2", "f32"), ("resnet50", None), ("resnet18", None), ("mobilenetv2", "f32"),
        ("densenet121", None), ("googlenet", None)]   # ... and two whose schedules fold nodes (concatenations in place, absorbed affine nodes)


def _setup(batch):
    import torch
    import paper_2410_21120_amd as fi
    members, specs, keep = [], [], []
    for i, (f, act) in enumerate(FAMS):
        m = zoo.FAMILIES[f](hw=HW)
        blob = gen.make_blob(m, 1000 + i)
        sp, k = fi.make_spec(m, blob.ctypes.data, blob.nbytes, act_dtype=act)
        members.append((m, blob, act))
        specs.append(sp)
        keep.append((k, blob))
    x = gen.make_input(7, batch, 3, HW, HW, "normal", "bf16")
    xin = torch.from_numpy(gen.to_nhwc_storage(x, "bf16").view(np.int16)).cuda()
    outs = [torch.full((batch, 1000), float("nan"), dtype=torch.float32, device="cuda:0") for _ in FAMS]
    return fi, torch, members, specs, keep, x, xin, outs


def test_round_robin_outputs_equal_each_model_alone():
    from tests import harness
    fi, torch, members, specs, keep, x, xin, outs = _setup(3)
    alone = []
    for mb in members:
        g = harness.GpuDag([mb], 3)
        try:
            alone.append(g.run(x)[0])
        finally:
            g.close()
    alloc = fi.TorchAllocators("cuda:0")
    opts = fi.make_opts(3, alloc)
    single = [fi.fi_footprint([sp], opts).device_bytes for sp in specs]
    budget = max(single) + 2 * min(single)
    group_of, n_groups = fi.fi_partition(specs, opts, budget)
    assert n_groups >= 2
    stream = torch.cuda.current_stream().cuda_stream
    for overlap in (False, True):
        for o in outs:
            o.fill_(float("nan"))
        torch.cuda.synchronize()
        st = fi.fi_round_robin(specs, opts, group_of, n_groups, 3, 2, overlap, xin.data_ptr(), 3, [o.data_ptr() for o in outs], stream)
        torch.cuda.synchronize()
        assert (st.n_groups, st.n_loads, st.n_runs) == (n_groups, 2 * n_groups, 2 * n_groups * 3)
        largest_pair = max(fi.fi_footprint([sp for sp, g in zip(specs, group_of) if g in (k, (k + 1) % n_groups)], opts).device_bytes
                           for k in range(n_groups))
        assert st.peak_device_bytes <= (2 * budget if overlap else budget)
        assert overlap or st.peak_device_bytes <= largest_pair
        for i, o in enumerate(outs):
            assert np.array_equal(o.cpu().numpy(), alone[i]), f"model {i}, overlap={overlap}"
        if overlap:   # what the scheduler left in every model's buffer, against the oracle run on that model alone
            for i, (m, blob, act) in enumerate(members):
                harness.check_against_oracle(f"{FAMS[i][0]}[{i}] after round robin", m, blob, act, x, outs[i].cpu().numpy())
    # one batch holding everything stays resident: a single load
    everything = fi.fi_footprint(specs, opts).device_bytes
    g1, n1 = fi.fi_partition(specs, opts, everything)
    st = fi.fi_round_robin(specs, opts, g1, n1, 2, 3, True, xin.data_ptr(), 3, [o.data_ptr() for o in outs], stream)
    torch.cuda.synchronize()
    assert (n1, st.n_loads, st.n_runs) == (1, 1, 6)
    for i, o in enumerate(outs):
        assert np.array_equal(o.cpu().numpy(), alone[i])
    assert not alloc.live or all(not t.is_cuda for t in alloc.live.values())  # nothing left on the device


def test_round_robin_argument_and_budget_errors():
    fi, torch, members, specs, keep, x, xin, outs = _setup(2)
    alloc = fi.TorchAllocators("cuda:0")
    opts = fi.make_opts(2, alloc)
    stream = torch.cuda.current_stream().cuda_stream
    ptrs = [o.data_ptr() for o in outs]
    with pytest.raises(fi.FiError) as e:
        fi.fi_round_robin(specs, opts, [0, 0, 2, 2, 2, 2], 3, 1, 1, False, xin.data_ptr(), 2, ptrs, stream)   # batch 1 is empty
    assert e.value.status == fi.FI_EINVAL
    with pytest.raises(fi.FiError) as e:
        fi.fi_round_robin(specs, opts, [0] * 6, 1, 0, 1, False, xin.data_ptr(), 2, ptrs, stream)              # no iterations
    assert e.value.status == fi.FI_EINVAL
    both = fi.fi_footprint(specs[:3], opts).device_bytes
    tight = fi.make_opts(2, alloc, max_device_bytes=both)
    with pytest.raises(fi.FiError) as e:   # each half fits the cap, two resident halves do not
        fi.fi_round_robin(specs, tight, [0, 0, 0, 1, 1, 1], 2, 1, 1, True, xin.data_ptr(), 2, ptrs, stream)
    assert e.value.status == fi.FI_EBUDGET
