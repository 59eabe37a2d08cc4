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
