"""Per-kernel GPU parity against the CPU oracle on small seeded shapes that span
several tiles and ragged tails (odd sizes, stride 2, padding edges, channel
counts that are not multiples of the tile)."""
import numpy as np
import pytest

from workloads import gen, zoo

pytestmark = pytest.mark.gpu

BF16_TOL = 1e-2   # relative L2 vs the fp32-activation oracle (mode F)
F32_TOL = 1e-4




def _run_case(model, seed, batch, act_dtype=None, tol=None, bias_std=0.1):
    from tests import harness
    model.shapes()
    blob = gen.make_blob(model, seed, bias_std=bias_std)
    x = gen.make_input(seed + 1, batch, model.in_c, model.in_h, model.in_w, "normal", model.dtype)
    g = harness.GpuDag([(model, blob, act_dtype)], batch)
    try:
        y = g.run(x)[0]
    finally:
        g.close()
    wide = (model.dtype == "f32") or act_dtype == "f32"
    ref_f = harness.oracle_nhwc(model, blob, x, False)
    assert y.shape == ref_f.shape
    assert np.isfinite(y).all()
    e = harness.rel_l2(y, ref_f)
    lim = tol if tol is not None else (F32_TOL if wide else BF16_TOL)
    assert e <= lim, f"rel L2 {e} > {lim}"
    if not wide:
        ref_s = harness.oracle_nhwc(model, blob, x, True)
        assert harness.rel_l2(y, ref_s) <= 2e-3
        ex = harness.elem_excess(y, ref_s, harness.ELEM_C_BF16)
    else:
        ex = harness.elem_excess(y, ref_f, harness.ELEM_C_F32)
    assert ex <= 1.0, f"an element is {ex:.2f}x its bound away from the oracle"
    return e


CONV_CASES = [  # cin, cout, k, stride, pad, H, W, batch
    (3, 16, 3, 1, 1, 32, 32, 1), (3, 64, 7, 2, 3, 37, 41, 2), (16, 24, 1, 1, 0, 17, 19, 3), (24, 144, 1, 1, 0, 28, 28, 2),
    (64, 64, 3, 1, 1, 14, 14, 2), (32, 160, 3, 2, 1, 15, 15, 3), (128, 256, 3, 2, 1, 9, 9, 2), (72, 40, 3, 1, 0, 11, 13, 1),
    (256, 512, 1, 2, 0, 14, 14, 2), (8, 8, 3, 1, 1, 5, 5, 1), (320, 1280, 1, 1, 0, 7, 7, 2), (64, 192, 3, 1, 1, 56, 56, 1),
    (3, 64, 11, 4, 2, 67, 71, 2), (64, 192, 5, 1, 2, 27, 27, 2), (16, 32, 15, 1, 7, 19, 17, 1),   # large kernels (up to 15x15)
]


@pytest.mark.parametrize("case", CONV_CASES)
@pytest.mark.parametrize("mode", ["bf16", "bf16_wide", "f32"])
def test_conv_relu(case, mode):
    cin, cout, k, s, p, h, w, b = case
    dtype = "f32" if mode == "f32" else "bf16"
    m = zoo.Model("c", dtype, cin, h, w)
    m.add(zoo.CONV, -1, cin=cin, cout=cout, k=k, stride=s, pad=p, act=zoo.RELU)
    _run_case(m, 100 + cin + cout, b, act_dtype="f32" if mode == "bf16_wide" else None)


def test_long_reductions_in_small_launches_keep_their_bits():
    """ResNet-50's last stage in isolation: a 3x3 over 512 channels and a 1x1 over 2048 at 7x7, batch 32, bring 52
    workgroups each and take the 128x128 tile with three reduction tiles in flight.  At batch 96 the same layers bring
    148 workgroups and take the plain tile: the first 32 images must come out with the same bits (the reduction order
    does not depend on the prefetch depth), and meet the oracle."""
    from tests import harness
    m = zoo.Model("stage4", "bf16", 512, 7, 7)
    a = m.add(zoo.CONV, -1, cin=512, cout=512, k=3, stride=1, pad=1, act=zoo.RELU)
    a = m.add(zoo.CONV, a, cin=512, cout=2048, k=1, stride=1, pad=0, act=zoo.RELU)
    a = m.add(zoo.CONV, a, cin=2048, cout=512, k=1, stride=1, pad=0, act=zoo.RELU)
    m.add(zoo.CONV, a, cin=512, cout=24, k=1, stride=1, pad=0, act=zoo.NONE)
    m.shapes()
    blob = gen.make_blob(m, 777)
    x = gen.make_input(778, 96, 512, 7, 7, "normal", "bf16")
    outs = {}
    for batch in (32, 96, 31):   # (31: a ragged last tile under the deep prefetch)
        g = harness.GpuDag([(m, blob, None)], batch)
        try:
            outs[batch] = g.run(x[:batch])[0]
        finally:
            g.close()
    assert np.isfinite(outs[32]).all()
    assert np.array_equal(outs[32], outs[96][:32]) and np.array_equal(outs[31], outs[96][:31])
    harness.check_against_oracle("last-stage layers, deep prefetch", m, blob, None, x[:32], outs[32], rows=[0, 7, 31])


@pytest.mark.parametrize("case", [(128, 128, 3, 1, 1, 127, 129, 4),   # 256x128 tile: long reduction, ragged last tile
                                  (64, 64, 3, 1, 1, 127, 129, 4),     # 256x64 tile: narrow, long reduction
                                  (256, 128, 1, 1, 0, 127, 129, 4)])  # 128x128 tile, pointwise prologue
def test_conv_large_tiles_bf16(case):
    """Shapes large enough (>= 256 workgroups) for the planner to pick the 256-row tiles."""
    import paper_2410_21120_amd as fi
    from tests import harness
    cin, cout, k, s, p, h, w, b = case
    m = zoo.Model("t", "bf16", cin, h, w)
    m.add(zoo.CONV, -1, cin=cin, cout=cout, k=k, stride=s, pad=p, act=zoo.RELU)
    m.shapes()
    blob = gen.make_blob(m, 300 + cin)
    g = harness.GpuDag([(m, blob, None)], b)
    try:
        names = [L.name.decode() for L in g.dag.launches()]
    finally:
        g.close()
    want = "conv_mfma_256x128" if (cin, cout) == (128, 128) else "conv_mfma_256x64" if cin == 64 else "conv_mfma_128x128"
    assert want in names, names
    _run_case(m, 300 + cin, b)


@pytest.mark.parametrize("mode", ["bf16", "bf16_wide", "f32"])
@pytest.mark.parametrize("act", [zoo.NONE, zoo.RELU, zoo.RELU6])
def test_conv_residual_and_activation(mode, act):
    dtype = "f32" if mode == "f32" else "bf16"
    m = zoo.Model("r", dtype, 16, 13, 13)
    a = m.add(zoo.CONV, -1, cin=16, cout=40, k=3, stride=1, pad=1, act=zoo.RELU)
    b = m.add(zoo.CONV, a, cin=40, cout=40, k=1, stride=1, pad=0, act=zoo.NONE)
    m.add(zoo.CONV, b, cin=40, cout=40, k=3, stride=1, pad=1, act=act, residual=a)
    _run_case(m, 7, 2, act_dtype="f32" if mode == "bf16_wide" else None)


@pytest.mark.parametrize("case", [(32, 3, 1, 1, 20, 20, 2), (96, 3, 2, 1, 15, 17, 2), (144, 3, 1, 1, 7, 7, 3), (24, 3, 2, 1, 9, 9, 1),
                                  (72, 5, 2, 2, 21, 19, 2), (120, 5, 1, 2, 14, 14, 2)])
@pytest.mark.parametrize("mode", ["bf16", "bf16_wide", "f32"])
def test_depthwise(case, mode):
    c, k, s, p, h, w, b = case
    dtype = "f32" if mode == "f32" else "bf16"
    m = zoo.Model("d", dtype, c, h, w)
    m.add(zoo.DWCONV, -1, cin=c, cout=c, k=k, stride=s, pad=p, act=zoo.RELU6)
    _run_case(m, 200 + c, b, act_dtype="f32" if mode == "bf16_wide" else None)


@pytest.mark.parametrize("case", [(64, 3, 2, 1, 23, 23, 2), (16, 2, 2, 0, 32, 32, 1), (24, 2, 2, 0, 15, 17, 3)])
@pytest.mark.parametrize("mode", ["bf16", "f32"])
def test_maxpool_exact(case, mode):
    """Pooling moves values without arithmetic: the result is bit-exact."""
    from tests import harness
    c, k, s, p, h, w, b = case
    m = zoo.Model("p", mode, c, h, w)
    m.add(zoo.MAXPOOL, -1, k=k, stride=s, pad=p)
    m.shapes()
    blob = np.zeros(64, np.uint8)
    x = -np.abs(gen.make_input(3, b, c, h, w, "normal", mode)) - 1.0  # all negative: padding must not win
    if mode == "bf16":
        x = gen.bf16_to_f32(gen.bf16_bits(x)).reshape(x.shape)
    g = harness.GpuDag([(m, blob)], b)
    try:
        y = g.run(x)[0]
    finally:
        g.close()
    assert np.array_equal(y, harness.oracle_nhwc(m, blob, x, False))


@pytest.mark.parametrize("case", [(64, 1, 9, 11, 2), (24, 1, 5, 2, 3), (40, 0, 7, 6, 1), (192, 1, 28, 28, 4), (8, 1, 1, 1, 2), (16, 1, 3, 13, 1)])  # C, pad, H, W, batch
def test_maxpool_3x3_stride1_inside_the_arena_is_exact(case):
    """The 3x3 stride-1 max pool of an Inception branch (bf16 tensors between other nodes: four outputs per thread),
    widths that are not multiples of four, with and without padding, all-negative inputs so that padding must not win."""
    from tests import harness
    c, p, h, w, b = case
    m = zoo.Model("p3", "bf16", c, h, w)
    a = m.add(zoo.MAXPOOL, -1, k=1, stride=1, pad=0)
    a = m.add(zoo.MAXPOOL, a, k=3, stride=1, pad=p)
    m.add(zoo.MAXPOOL, a, k=1, stride=1, pad=0)
    m.shapes()
    blob = np.zeros(64, np.uint8)
    x = -np.abs(gen.make_input(4 + c, b, c, h, w, "normal", "bf16")) - 1.0
    x = gen.bf16_to_f32(gen.bf16_bits(x)).reshape(x.shape)
    g = harness.GpuDag([(m, blob)], b)
    try:
        y = g.run(x)[0]
        names = [L.name.decode() for L in g.dag.launches()]
    finally:
        g.close()
    assert names.count("maxpool") == 3
    assert np.array_equal(y, harness.oracle_nhwc(m, blob, x, False))


@pytest.mark.parametrize("case", [(128, 128, 1, 7, 1, 3, 17, 17, 2), (128, 192, 7, 1, 1, 3, 17, 17, 2), (384, 384, 1, 3, 1, 1, 8, 8, 2),
                                  (384, 384, 3, 1, 1, 1, 8, 8, 2), (24, 40, 3, 1, 2, 1, 15, 13, 1), (3, 16, 1, 5, 1, 2, 20, 21, 2),
                                  (16, 16, 5, 2, 2, 2, 19, 18, 1)])   # cin, cout, kh, kw, stride, pad, H, W, batch
@pytest.mark.parametrize("mode", ["bf16", "bf16_wide", "f32"])
def test_rectangular_kernels(case, mode):
    """1 x n, n x 1 and other rectangular kernels; padding only along the dimensions the kernel extends over."""
    cin, cout, kh, kw, s, p, h, w, b = case
    dtype = "f32" if mode == "f32" else "bf16"
    m = zoo.Model("rect", dtype, cin, h, w)
    m.add(zoo.CONV, -1, cin=cin, cout=cout, k=kh, kw=kw, stride=s, pad=p, act=zoo.RELU)
    _run_case(m, 1500 + cin + kh * 16 + kw, b, act_dtype="f32" if mode == "bf16_wide" else None)


@pytest.mark.parametrize("case", [(128, 128, 32, 3, 1, 1, 14, 14, 2), (64, 96, 4, 3, 2, 1, 15, 17, 2), (48, 48, 48, 3, 1, 1, 9, 9, 1),
                                  (32, 64, 2, 1, 1, 0, 12, 12, 3), (256, 256, 32, 3, 2, 1, 28, 28, 1),
                                  # channel strides that whole reduction tiles divide: a column tile walks its own groups' channels only.
                                  # One group per 64-channel tile; two groups per tile; groups wider than a tile (tiles straddle them);
                                  # the 256-row and the 128-row tile; a 1x1 and a 5x5 filter
                                  (192, 192, 3, 3, 1, 1, 13, 11, 2), (256, 128, 4, 3, 2, 1, 14, 14, 2), (128, 320, 2, 3, 1, 1, 9, 10, 2),
                                  (128, 128, 32, 3, 1, 1, 56, 56, 24), (128, 128, 32, 3, 1, 1, 32, 32, 16), (256, 192, 8, 1, 1, 0, 12, 12, 2),
                                  (64, 128, 2, 5, 1, 2, 11, 11, 1)])  # cin, cout, groups, k, stride, pad, H, W, batch
@pytest.mark.parametrize("mode", ["bf16", "bf16_wide", "f32"])
def test_grouped_conv(case, mode):
    """Grouped convolution (each output channel sees its own group of input channels), up to one group per channel."""
    cin, cout, groups, k, s, p, h, w, b = case
    dtype = "f32" if mode == "f32" else "bf16"
    m = zoo.Model("gc", dtype, cin, h, w)
    m.add(zoo.CONV, -1, cin=cin, cout=cout, k=k, stride=s, pad=p, act=zoo.RELU, groups=groups)
    _run_case(m, 700 + cin + groups, b, act_dtype="f32" if mode == "bf16_wide" else None)


@pytest.mark.parametrize("case", [(16, 24, 13, 15), (8, 8, 6, 6), (20, 12, 9, 7), (64, 64, 28, 28)])   # channels of the two sources, H, W
@pytest.mark.parametrize("mode", ["bf16", "bf16_wide", "f32"])
def test_concat_of_two_branches(case, mode):
    """Concatenation followed by a convolution that mixes all channels: vector path (first source a multiple
    of 8 channels) and element path (20 + 12), padded channel strides on both sides."""
    ca, cb, h, w = case
    dtype = "f32" if mode == "f32" else "bf16"
    m = zoo.Model("cat", dtype, 8, h, w)
    a = m.add(zoo.CONV, -1, cin=8, cout=ca, k=1, stride=1, pad=0, act=zoo.RELU)
    b = m.add(zoo.CONV, -1, cin=8, cout=cb, k=3, stride=1, pad=1, act=zoo.RELU)
    c = m.add(zoo.CONCAT, a, residual=b)
    m.add(zoo.CONV, c, cin=ca + cb, cout=10, k=1, stride=1, pad=0, act=zoo.NONE)
    _run_case(m, 500 + ca + cb, 2, act_dtype="f32" if mode == "bf16_wide" else None)


def test_concat_as_output_node_is_exact():
    """A concat that is the member's output copies values: the fp32 result equals the oracle's exactly in
    storage-rounding mode (both sides hold the same bf16 values)."""
    from tests import harness
    m = zoo.Model("cat_out", "bf16", 8, 8, 10)
    a = m.add(zoo.MAXPOOL, -1, k=3, stride=2, pad=0, ceil=True)
    b = m.add(zoo.MAXPOOL, -1, k=2, stride=2, pad=0, ceil=True)
    m.add(zoo.CONCAT, a, residual=b)
    m.shapes()
    blob = np.zeros(64, np.uint8)   # no weighted node
    x = gen.make_input(3, 2, 8, 8, 10, "normal", "bf16")
    g = harness.GpuDag([(m, blob, None)], 2)
    try:
        y = g.run(x)[0]
    finally:
        g.close()
    assert np.array_equal(y, harness.oracle_nhwc(m, blob, x, True))


@pytest.mark.parametrize("case", [(64, 3, 2, 0, 23, 24, 2), (16, 3, 2, 0, 8, 8, 1), (24, 3, 1, 1, 14, 14, 2), (40, 2, 2, 0, 7, 9, 3), (8, 2, 2, 1, 5, 5, 1)])
@pytest.mark.parametrize("mode", ["bf16", "f32"])
def test_maxpool_ceil_mode_exact(case, mode):
    """Pooling whose size rounds up: windows hang over the far edge; those taps never win (all-negative input)."""
    from tests import harness
    c, k, s, p, h, w, b = case
    m = zoo.Model("pc", mode, c, h, w)
    m.add(zoo.MAXPOOL, -1, k=k, stride=s, pad=p, ceil=True)
    m.shapes()
    blob = np.zeros(64, np.uint8)   # no weighted node
    x = -np.abs(gen.make_input(3, b, c, h, w, "normal", mode)) - 0.5
    if mode == "bf16":
        x = gen.bf16_to_f32(gen.bf16_bits(x)).reshape(x.shape)
    g = harness.GpuDag([(m, blob, None)], b)
    try:
        y = g.run(x)[0]
    finally:
        g.close()
    ref = harness.oracle_nhwc(m, blob, x, False)
    assert y.shape == ref.shape and np.array_equal(y, ref)


@pytest.mark.parametrize("case", [(64, 2, 2, 0, 28, 28, 2), (24, 3, 1, 1, 9, 11, 2), (40, 3, 2, 1, 15, 14, 1), (8, 5, 1, 2, 7, 7, 3),
                                  (192, 3, 1, 1, 17, 17, 3), (16, 3, 1, 0, 6, 5, 2)])
@pytest.mark.parametrize("mode", ["bf16", "bf16_wide", "f32"])
def test_avgpool_between_convs(case, mode):
    """Window average pooling (divisor = window area, zero padding counted) between two convolutions."""
    c, k, s, p, h, w, b = case
    dtype = "f32" if mode == "f32" else "bf16"
    m = zoo.Model("ap", dtype, 8, h, w)
    a = m.add(zoo.CONV, -1, cin=8, cout=c, k=1, stride=1, pad=0, act=zoo.RELU)
    a = m.add(zoo.AVGPOOL, a, k=k, stride=s, pad=p)
    m.add(zoo.CONV, a, cin=c, cout=12, k=1, stride=1, pad=0, act=zoo.NONE)
    _run_case(m, 900 + c + k, b, act_dtype="f32" if mode == "bf16_wide" else None)


@pytest.mark.parametrize("act", [zoo.HARDSWISH, zoo.HARDSIGMOID, zoo.SILU, zoo.SIGMOID])
@pytest.mark.parametrize("mode", ["bf16", "bf16_wide", "f32"])
def test_smooth_activations_in_every_epilogue(act, mode):
    """Hard-swish, hard-sigmoid, SiLU and sigmoid after an MFMA / direct convolution, a split-K convolution
    (finished by the reduce kernel), a depthwise convolution and a small-batch FC."""
    dtype = "f32" if mode == "f32" else "bf16"
    m = zoo.Model("acts", dtype, 16, 12, 12)
    a = m.add(zoo.CONV, -1, cin=16, cout=40, k=3, stride=1, pad=1, act=act)
    a = m.add(zoo.DWCONV, a, cin=40, cout=40, k=3, stride=2, pad=1, act=act)
    a = m.add(zoo.CONV, a, cin=40, cout=64, k=3, stride=1, pad=1, act=act)      # 6x6 outputs, K = 360: split-K at this size
    a = m.add(zoo.GAP, a)
    m.add(zoo.FC, a, cin=64, cout=20, act=act)
    _run_case(m, 1100, 2, act_dtype="f32" if mode == "bf16_wide" else None)


@pytest.mark.parametrize("case", [(64, 16, 9, 11, 2), (24, 8, 7, 7, 3), (120, 32, 14, 14, 1)])   # channels, squeeze width, H, W, batch
@pytest.mark.parametrize("mode", ["bf16", "bf16_wide", "f32"])
def test_squeeze_excite_block(case, mode):
    """global average -> FC (ReLU) -> FC (hard sigmoid) -> per-channel scaling of the block's tensor -> 1x1 projection."""
    c, sq, h, w, b = case
    dtype = "f32" if mode == "f32" else "bf16"
    m = zoo.Model("se", dtype, 8, h, w)
    x = m.add(zoo.CONV, -1, cin=8, cout=c, k=1, stride=1, pad=0, act=zoo.HARDSWISH)
    g = m.add(zoo.GAP, x)
    g = m.add(zoo.FC, g, cin=c, cout=sq, act=zoo.RELU)
    g = m.add(zoo.FC, g, cin=sq, cout=c, act=zoo.HARDSIGMOID)
    y = m.add(zoo.MUL, x, residual=g)
    m.add(zoo.CONV, y, cin=c, cout=16, k=1, stride=1, pad=0, act=zoo.NONE)
    _run_case(m, 1200 + c, b, act_dtype="f32" if mode == "bf16_wide" else None)


@pytest.mark.parametrize("mode", ["bf16", "bf16_wide", "f32"])
def test_slice_branch_concat_shuffle_unit(mode):
    """One ShuffleNet-V2-style unit: half of the channels kept, the other half through 1x1 -> depthwise -> 1x1,
    concatenated and shuffled in two groups; odd half-width (29) so the element paths with ragged padding run."""
    dtype = "f32" if mode == "f32" else "bf16"
    m = zoo.Model("shuf", dtype, 8, 10, 9)
    x = m.add(zoo.CONV, -1, cin=8, cout=58, k=1, stride=1, pad=0, act=zoo.RELU)
    a = m.add(zoo.SLICE, x, first=0, cout=29)
    b = m.add(zoo.SLICE, x, first=29, cout=29)
    b = m.add(zoo.CONV, b, cin=29, cout=29, k=1, stride=1, pad=0, act=zoo.RELU)
    b = m.add(zoo.DWCONV, b, cin=29, cout=29, k=3, stride=1, pad=1, act=zoo.NONE)
    y = m.add(zoo.CONCAT, a, residual=b)
    y = m.add(zoo.SHUFFLE, y, groups=2)
    m.add(zoo.CONV, y, cin=58, cout=12, k=1, stride=1, pad=0, act=zoo.NONE)
    _run_case(m, 1300, 2, act_dtype="f32" if mode == "bf16_wide" else None)


@pytest.mark.parametrize("case", [(16, 8, 3, 9, 7, 2), (64, 32, 4, 28, 28, 4), (24, 16, 2, 5, 5, 1)])   # first width, growth, layers, H, W, batch
@pytest.mark.parametrize("mode", ["bf16", "bf16_wide"])
def test_dense_block_concatenations(case, mode):
    """A DenseNet-style block: every layer normalises (per-channel affine + ReLU) everything concatenated so far and appends
    `growth` new channels.  With bf16 activations the new channels are written straight into the block's final tensor and
    the affine nodes read its prefixes with that tensor's channel stride; with fp32 activations every concatenation copies."""
    c0, growth, layers, h, w, b = case
    m = zoo.Model("dense", "bf16", 8, h, w)
    t = m.add(zoo.CONV, -1, cin=8, cout=c0, k=3, stride=1, pad=1, act=zoo.RELU)
    c = c0
    for _ in range(layers):
        a = m.add(zoo.DWCONV, t, cin=c, cout=c, k=1, stride=1, pad=0, act=zoo.RELU)
        a = m.add(zoo.CONV, a, cin=c, cout=4 * growth, k=1, stride=1, pad=0, act=zoo.RELU)
        a = m.add(zoo.CONV, a, cin=4 * growth, cout=growth, k=3, stride=1, pad=1, act=zoo.NONE)
        t = m.add(zoo.CONCAT, t, residual=a)
        c += growth
    t = m.add(zoo.DWCONV, t, cin=c, cout=c, k=3, stride=2, pad=1, act=zoo.RELU)
    t = m.add(zoo.GAP, t)
    m.add(zoo.FC, t, cin=c, cout=10)
    _run_case(m, 1700 + c0, b, act_dtype="f32" if mode == "bf16_wide" else None)


@pytest.mark.parametrize("mode", ["bf16", "bf16_wide"])
def test_reduction_module_concatenations(mode):
    """An Inception-style reduction module: a strided convolution, a two-convolution branch, a strided max pool and an
    average pool of the same input, joined by nested concatenations (pool outputs and convolution outputs side by side in
    one tensor), then read by a dense convolution."""
    m = zoo.Model("red", "bf16", 8, 17, 15)
    x = m.add(zoo.CONV, -1, cin=8, cout=48, k=1, stride=1, pad=0, act=zoo.RELU)
    b1 = m.add(zoo.CONV, x, cin=48, cout=40, k=3, stride=2, pad=0, act=zoo.RELU)
    b2 = m.add(zoo.CONV, x, cin=48, cout=16, k=1, stride=1, pad=0, act=zoo.RELU)
    b2 = m.add(zoo.CONV, b2, cin=16, cout=24, k=3, stride=2, pad=0, act=zoo.RELU)
    b3 = m.add(zoo.MAXPOOL, x, k=3, stride=2, pad=0)
    b4 = m.add(zoo.AVGPOOL, x, k=3, stride=2, pad=0)
    y = m.add(zoo.CONCAT, b1, residual=b2)
    y = m.add(zoo.CONCAT, y, residual=b3)
    y = m.add(zoo.CONCAT, y, residual=b4)
    m.add(zoo.CONV, y, cin=160, cout=12, k=3, stride=1, pad=1, act=zoo.NONE)
    _run_case(m, 1800, 3, act_dtype="f32" if mode == "bf16_wide" else None)


@pytest.mark.parametrize("case", [(64, 16, 24, 2), (64, 8, 20, 4), (48, 0, 48, 3), (120, 56, 64, 2), (24, 0, 24, 3), (64, 32, 32, 1)])  # C, first, width, shuffle groups
def test_slice_and_shuffle_inside_the_arena_are_exact(case):
    """Channel slices at vector-aligned and unaligned offsets, widths that do and do not fill whole 8-channel vectors,
    shuffles in 1..4 groups, all between other nodes (bf16 tensors in the arena: the 8-channel form of the gather):
    values only move, so the result equals the oracle's bit for bit."""
    from tests import harness
    c, first, width, groups = case
    m = zoo.Model("gath", "bf16", c, 6, 5)
    a = m.add(zoo.MAXPOOL, -1, k=1, stride=1, pad=0)
    a = m.add(zoo.SLICE, a, first=first, cout=width)
    a = m.add(zoo.SHUFFLE, a, groups=groups)
    m.add(zoo.MAXPOOL, a, k=1, stride=1, pad=0)
    m.shapes()
    x = gen.make_input(5 + c, 3, c, 6, 5, "normal", "bf16")
    blob = np.zeros(64, np.uint8)
    g = harness.GpuDag([(m, blob, None)], 3)
    try:
        y = g.run(x)[0]
    finally:
        g.close()
    assert np.array_equal(y, harness.oracle_nhwc(m, blob, x, True))


def test_shuffle_as_output_node_is_exact():
    from tests import harness
    m = zoo.Model("shuf_out", "bf16", 24, 5, 7)
    a = m.add(zoo.MAXPOOL, -1, k=1, stride=1, pad=0)
    a = m.add(zoo.SLICE, a, first=6, cout=12)
    m.add(zoo.SHUFFLE, a, groups=4)
    m.shapes()
    x = gen.make_input(3, 2, 24, 5, 7, "normal", "bf16")
    blob = np.zeros(64, np.uint8)
    g = harness.GpuDag([(m, blob, None)], 2)
    try:
        y = g.run(x)[0]
    finally:
        g.close()
    assert np.array_equal(y, harness.oracle_nhwc(m, blob, x, True))


@pytest.mark.parametrize("mode", ["bf16", "bf16_wide", "f32"])
def test_gap_fc_softmax_chain(mode):
    dtype = "f32" if mode == "f32" else "bf16"
    m = zoo.Model("g", dtype, 24, 7, 9)
    a = m.add(zoo.GAP, -1)
    a = m.add(zoo.FC, a, cin=24, cout=50, act=zoo.RELU)
    a = m.add(zoo.FC, a, cin=50, cout=10)
    m.add(zoo.SOFTMAX, a)
    e = _run_case(m, 31, 5, act_dtype="f32" if mode == "bf16_wide" else None)
    assert e < 5e-3


def test_fc_on_spatial_input_bf16():
    """FC over a flattened C,H,W tensor (the 25088-input layer shape, scaled down)."""
    m = zoo.Model("f", "bf16", 40, 7, 7)
    m.add(zoo.FC, -1, cin=40 * 49, cout=130, act=zoo.RELU)
    _run_case(m, 5, 8)


@pytest.mark.parametrize("mode", ["bf16", "bf16_wide"])
@pytest.mark.parametrize("batch", [33, 70])
def test_fc_batches_above_32_and_residual(batch, mode):
    """The FC kernel takes 32 images per pass: batches that need two and three passes (the last one ragged), a
    feature count that is not a multiple of 32, and an FC that adds a residual."""
    m = zoo.Model("f", "bf16", 24, 5, 3)
    a = m.add(zoo.FC, -1, cin=24 * 15, cout=77, act=zoo.RELU)
    b = m.add(zoo.FC, a, cin=77, cout=77, act=zoo.NONE)
    c = m.add(zoo.FC, b, cin=77, cout=77, act=zoo.RELU, residual=a)
    m.add(zoo.FC, c, cin=77, cout=1000)
    _run_case(m, 77, batch, act_dtype="f32" if mode == "bf16_wide" else None)


def test_batch_smaller_than_max_batch():
    from tests import harness
    m = zoo.resnet18(hw=64)
    blob = gen.make_blob(m, 1000)
    x = gen.make_input(7, 4, 3, 64, 64, "normal", "bf16")
    g = harness.GpuDag([(m, blob)], 4)
    try:
        full = g.run(x)[0]
        part = g.run(x[:3])[0]
        one = g.run(x[2:3])[0]
    finally:
        g.close()
    assert np.array_equal(full[:3], part) and np.array_equal(full[2:3], one)
