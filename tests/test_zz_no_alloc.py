"""The entry point that allocates nothing (fi_run_static: split-K partial sums in the library's static device
array) against fi_run, through the C-ABI, on two calls in a row, the second with a smaller input: the same
kernels in the same order, so the same bits; and against the CPU oracle.  Runs last: the static array is shared
by every call on the GPU."""
import numpy as np
import pytest

from workloads import gen, zoo

pytestmark = pytest.mark.gpu


def test_run_static_equals_run_on_two_calls_in_a_row():
    import torch
    import paper_2410_21120_amd as fi
    from tests import harness
    hw = 64
    fams = [("resnet18", None), ("vgg16", None), ("resnet18", None), ("mobilenetv2", "f32")]
    mem = []
    for i, (f, act) in enumerate(fams):
        m = zoo.FAMILIES[f](hw=hw)
        mem.append((m, gen.make_blob(m, 6000 + i), act))
    g = harness.GpuDag(mem, 5)
    torch.cuda.synchronize()
    try:
        q = g.dag.query()
        names = [L.name.decode() for L in g.dag.launches()]
        assert q.workspace_bytes > 0 and "splitk_reduce" in names and "fc_splitk" in names   # the scratch buffer is really used
        for batch, seed in ((5, 61), (2, 62)):   # the second call is smaller and finds the first call's partial sums in the array
            x = gen.make_input(seed, batch, 3, hw, hw, "normal", "bf16")
            want = g.run(x)
            xin = torch.from_numpy(gen.to_nhwc_storage(x, "bf16").view(np.int16)).cuda()
            outs = [torch.full((batch, 1000), float("nan"), dtype=torch.float32, device="cuda:0") for _ in mem]
            torch.cuda.synchronize()
            before = torch.cuda.memory_stats()["allocation.all.allocated"]
            g.dag.run_static(xin.data_ptr(), batch, [o.data_ptr() for o in outs], g.stream)
            torch.cuda.synchronize()
            assert torch.cuda.memory_stats()["allocation.all.allocated"] == before   # nothing went through the allocator behind the handle
            for i, (m, blob, act) in enumerate(mem):
                y = outs[i].cpu().numpy()
                assert np.array_equal(y, want[i]), f"batch {batch}, member {i}: fi_run_static differs from fi_run"
                harness.check_against_oracle(f"{fams[i][0]}[{i}] batch {batch}", m, blob, act, x, y)
    finally:
        g.close()


def test_run_static_refuses_a_workspace_larger_than_the_array():
    import paper_2410_21120_amd as fi
    from tests import harness
    # several VGG-16 at batch 64: every member's FC layers keep 16 slices x 64 images x 4096 features of partial sums
    mem = []
    m = zoo.FAMILIES["vgg16"](hw=32)
    blob = gen.make_blob(m, 6100)
    g = None
    for n in (4, 16):
        mem = [(m, blob, None)] * n
        g = harness.GpuDag(mem, 64)
        if g.dag.query().workspace_bytes > (32 << 20):
            break
        g.close()
        g = None
    assert g is not None, "no test DAG exceeds the static array"
    try:
        import torch
        x = gen.make_input(63, 1, 3, 32, 32, "normal", "bf16")
        xin = torch.from_numpy(gen.to_nhwc_storage(x, "bf16").view(np.int16)).cuda()
        outs = [torch.zeros((1, 1000), dtype=torch.float32, device="cuda:0") for _ in mem]
        with pytest.raises(fi.FiError) as e:
            g.dag.run_static(xin.data_ptr(), 1, [o.data_ptr() for o in outs], g.stream)
        assert e.value.status == fi.FI_EBUDGET
    finally:
        g.close()
