"""Pins for the CPU oracle: every layer function is checked against something
other than itself -- an independently formulated brute force, a library routine
in fp64, a closed form, or an algebraic invariant -- chosen so that a dropped
term, a wrong sign or index, or a transposed operand fails at least one test.
The paper prints no worked numeric example (no logits, no tensors), so the pins
are the mathematics of the layer definitions it delegates to a vendor library.
"""
import numpy as np
import pytest
import torch

import oracle

CASES = [  # (N, C, H, W, O, k, stride, pad)
    (1, 1, 5, 5, 1, 1, 1, 0), (2, 3, 7, 9, 4, 3, 1, 1), (2, 5, 9, 8, 3, 3, 2, 1), (1, 4, 9, 9, 2, 3, 2, 0),
    (1, 2, 9, 9, 3, 7, 2, 3), (2, 3, 8, 6, 5, 1, 2, 0), (1, 3, 6, 7, 2, 3, 1, 3), (1, 3, 11, 10, 4, 7, 1, 3),
]


def _scatter_conv(x, w, b, s, p):
    """Scatter form in fp64: every input pixel adds into the outputs it touches."""
    n, c, h, ww = x.shape
    o, _, k, _ = w.shape
    ho, wo = (h + 2 * p - k) // s + 1, (ww + 2 * p - k) // s + 1
    y = np.zeros((n, o, ho, wo), dtype=np.float64) + b.reshape(1, o, 1, 1).astype(np.float64)
    for ih in range(h):
        for iw in range(ww):
            for r in range(k):
                for t in range(k):
                    ni, nj = ih + p - r, iw + p - t
                    if ni % s or nj % s:
                        continue
                    i, j = ni // s, nj // s
                    if 0 <= i < ho and 0 <= j < wo:
                        y[:, :, i, j] += x[:, :, ih, iw].astype(np.float64) @ w[:, :, r, t].astype(np.float64).T
    return y


def _im2col_conv(x, w, b, s, p):
    """Explicit patch matrix times a library matmul in fp64."""
    n, c, h, ww = x.shape
    o, _, k, _ = w.shape
    xp = np.zeros((n, c, h + 2 * p, ww + 2 * p), dtype=np.float64)
    xp[:, :, p:p + h, p:p + ww] = x
    ho, wo = (h + 2 * p - k) // s + 1, (ww + 2 * p - k) // s + 1
    cols = np.empty((n, ho, wo, c * k * k), dtype=np.float64)
    for i in range(ho):
        for j in range(wo):
            cols[:, i, j, :] = xp[:, :, i * s:i * s + k, j * s:j * s + k].reshape(n, -1)
    y = cols.reshape(-1, c * k * k) @ w.reshape(o, -1).astype(np.float64).T + b.astype(np.float64)
    return y.reshape(n, ho, wo, o).transpose(0, 3, 1, 2)


@pytest.mark.parametrize("case", CASES)
def test_conv_vs_bruteforce_and_library(case, rng):
    n, c, h, ww, o, k, s, p = case
    x = rng.standard_normal((n, c, h, ww)).astype(np.float32)
    w = rng.standard_normal((o, c, k, k)).astype(np.float32)
    b = rng.standard_normal(o).astype(np.float32)
    y = oracle.conv2d(x, w, b, s, p)
    ys = _scatter_conv(x, w, b, s, p)
    yi = _im2col_conv(x, w, b, s, p)
    yl = torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(),
                                    torch.from_numpy(b).double(), stride=s, padding=p).numpy()
    assert y.shape == ys.shape == yi.shape == yl.shape
    for ref in (ys, yi, yl):
        assert np.abs(y - ref).max() <= 1e-5 * max(1.0, np.abs(ref).max())
    # the double-accumulation build is the same definition, tighter
    y64 = oracle.conv2d(x, w, b, s, p, f64=True)
    assert np.abs(y64 - yl).max() <= 2e-7 * max(1.0, np.abs(yl).max())


@pytest.mark.parametrize("case", [(2, 5, 9, 9, 3, 1, 1), (1, 6, 8, 7, 3, 2, 1), (1, 3, 9, 9, 3, 2, 0), (2, 4, 6, 6, 1, 1, 0)])
def test_depthwise_vs_library_and_per_channel_conv(case, rng):
    n, c, h, ww, k, s, p = case
    x = rng.standard_normal((n, c, h, ww)).astype(np.float32)
    w = rng.standard_normal((c, 1, k, k)).astype(np.float32)
    b = rng.standard_normal(c).astype(np.float32)
    y = oracle.dwconv2d(x, w, b, s, p)
    yl = torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(),
                                    torch.from_numpy(b).double(), stride=s, padding=p, groups=c).numpy()
    assert np.abs(y - yl).max() <= 1e-5 * max(1.0, np.abs(yl).max())
    # channel ch of a depthwise conv is a 1-in/1-out dense conv (brute force, scatter form)
    for ch in range(c):
        ys = _scatter_conv(x[:, ch:ch + 1], w[ch:ch + 1], b[ch:ch + 1], s, p)
        assert np.abs(y[:, ch:ch + 1] - ys).max() <= 1e-5 * max(1.0, np.abs(ys).max())


def test_delta_and_identity_kernels(rng):
    x = rng.standard_normal((2, 4, 6, 7)).astype(np.float32)
    zero = np.zeros(4, dtype=np.float32)
    w = np.zeros((4, 4, 3, 3), dtype=np.float32)
    for ch in range(4):
        w[ch, ch, 1, 1] = 1.0
    assert np.array_equal(oracle.conv2d(x, w, zero, 1, 1), x)  # centre delta: exact copy
    # off-centre delta (r=0, t=2): y[i,j] = x[i-1, j+1] with zero fill
    w2 = np.zeros_like(w)
    for ch in range(4):
        w2[ch, ch, 0, 2] = 1.0
    y = oracle.conv2d(x, w2, zero, 1, 1)
    exp = np.zeros_like(x)
    exp[:, :, 1:, :-1] = x[:, :, :-1, 1:]
    assert np.array_equal(y, exp)
    # 1x1 identity matrix
    w1 = np.eye(4, dtype=np.float32).reshape(4, 4, 1, 1)
    assert np.array_equal(oracle.conv2d(x, w1, zero, 1, 0), x)
    # a channel permutation via 1x1 (catches a transposed O/I index)
    perm = [2, 0, 3, 1]
    wp = np.zeros((4, 4, 1, 1), dtype=np.float32)
    for o, c in enumerate(perm):
        wp[o, c, 0, 0] = 1.0
    assert np.array_equal(oracle.conv2d(x, wp, zero, 1, 0), x[:, perm])
    # depthwise centre delta, and stride-2 sub-sampling
    wd = np.zeros((4, 1, 3, 3), dtype=np.float32)
    wd[:, 0, 1, 1] = 1.0
    assert np.array_equal(oracle.dwconv2d(x, wd, zero, 1, 1), x)
    assert np.array_equal(oracle.dwconv2d(x, wd, zero, 2, 1), x[:, :, ::2, ::2])
    assert np.array_equal(oracle.conv2d(x, w, zero, 2, 1), x[:, :, ::2, ::2])


def test_all_ones_closed_form():
    cin = 5
    x = np.ones((1, cin, 6, 8), dtype=np.float32)
    w = np.ones((2, cin, 3, 3), dtype=np.float32)
    y = oracle.conv2d(x, w, np.zeros(2, np.float32), 1, 1)
    assert np.all(y[:, :, 1:-1, 1:-1] == 9 * cin)
    assert np.all(y[:, :, 0, 1:-1] == 6 * cin) and np.all(y[:, :, 1:-1, 0] == 6 * cin)
    assert np.all(y[:, :, -1, 1:-1] == 6 * cin) and np.all(y[:, :, 1:-1, -1] == 6 * cin)
    for i, j in ((0, 0), (0, -1), (-1, 0), (-1, -1)):
        assert np.all(y[:, :, i, j] == 4 * cin)
    # bias is added once per output element
    y2 = oracle.conv2d(x, w, np.array([1.5, -2.0], np.float32), 1, 1)
    assert np.array_equal(y2[:, 0], y[:, 0] + 1.5) and np.array_equal(y2[:, 1], y[:, 1] - 2.0)


def test_linearity(rng):
    x1 = rng.standard_normal((1, 3, 8, 8)).astype(np.float32)
    x2 = rng.standard_normal((1, 3, 8, 8)).astype(np.float32)
    w = rng.standard_normal((4, 3, 3, 3)).astype(np.float32)
    z = np.zeros(4, np.float32)
    a, b = 0.75, -1.25
    lhs = oracle.conv2d(a * x1 + b * x2, w, z, 2, 1)
    rhs = a * oracle.conv2d(x1, w, z, 2, 1) + b * oracle.conv2d(x2, w, z, 2, 1)
    assert np.abs(lhs - rhs).max() < 1e-4


def test_batchnorm_fold_identity(rng):
    """Inference BN after a bias-free conv == conv with w*g/sqrt(v+eps) and bias beta - mu*g/sqrt(v+eps)."""
    x = rng.standard_normal((2, 3, 7, 7)).astype(np.float32)
    w = rng.standard_normal((5, 3, 3, 3)).astype(np.float32)
    g, beta, mu = (rng.standard_normal(5).astype(np.float32) for _ in range(3))
    var = rng.random(5).astype(np.float32) + 0.5
    eps = 1e-5
    y = oracle.conv2d(x, w, None, 1, 1)
    bn = g.reshape(1, 5, 1, 1) * (y - mu.reshape(1, 5, 1, 1)) / np.sqrt(var.reshape(1, 5, 1, 1) + eps) + beta.reshape(1, 5, 1, 1)
    sc = g / np.sqrt(var + eps)
    yf = oracle.conv2d(x, w * sc.reshape(5, 1, 1, 1), beta - mu * sc, 1, 1)
    assert np.abs(bn - yf).max() < 1e-4


def test_maxpool_closed_forms():
    h, w = 8, 10
    ramp = (np.arange(h)[:, None] * w + np.arange(w)[None, :]).astype(np.float32).reshape(1, 1, h, w)
    y = oracle.maxpool2d(ramp, 2, 2, 0)
    exp = ramp[:, :, 1::2, 1::2]  # max of each 2x2 window of an increasing ramp = its bottom-right tap
    assert np.array_equal(y, exp)
    # 3x3 stride 2 pad 1 on the ramp: window rows {2i-1..2i+1}, so max at (min(2i+1,h-1), min(2j+1,w-1))
    y3 = oracle.maxpool2d(ramp, 3, 2, 1)
    assert y3.shape == (1, 1, 4, 5)
    for i in range(4):
        for j in range(5):
            assert y3[0, 0, i, j] == ramp[0, 0, min(2 * i + 1, h - 1), min(2 * j + 1, w - 1)]
    # padding is -inf, not zero: an all-negative tensor stays negative
    neg = -np.ones((1, 2, 5, 5), dtype=np.float32) - np.arange(25, dtype=np.float32).reshape(5, 5)
    yn = oracle.maxpool2d(neg, 3, 2, 1)
    assert np.all(yn < 0) and yn[0, 0, 0, 0] == -1.0
    lib = torch.nn.functional.max_pool2d(torch.from_numpy(neg), 3, 2, 1).numpy()
    assert np.array_equal(yn, lib)
    # odd size, floor: 7 -> 3 with 2x2/2
    assert oracle.maxpool2d(np.zeros((1, 1, 7, 7), np.float32), 2, 2, 0).shape == (1, 1, 3, 3)


@pytest.mark.parametrize("case", [(12, 8, 4, 3, 1, 1), (16, 16, 2, 3, 2, 1), (6, 9, 3, 1, 1, 0), (8, 8, 8, 3, 1, 1), (10, 4, 1, 5, 2, 2)])
def test_grouped_conv_vs_per_group_dense_conv_and_library(case, rng):
    """A grouped convolution is G dense convolutions on channel slices laid side by side; one group is the
    dense convolution; as many groups as channels is the depthwise one; a library routine agrees."""
    import torch.nn.functional as F
    c, o, g, k, s, p = case
    x = rng.standard_normal((2, c, 9, 7)).astype(np.float32)
    w = rng.standard_normal((o, c // g, k, k)).astype(np.float32)
    b = rng.standard_normal(o).astype(np.float32)
    y = oracle.conv2d_grouped(x, w, b, g, s, p)
    cg, og = c // g, o // g
    parts = [oracle.conv2d(x[:, i * cg:(i + 1) * cg], w[i * og:(i + 1) * og], b[i * og:(i + 1) * og], s, p) for i in range(g)]
    assert np.array_equal(y, np.concatenate(parts, axis=1))
    ref = F.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(), torch.from_numpy(b).double(), s, p, 1, g).numpy()
    assert np.abs(y - ref).max() <= 1e-4 * max(1.0, np.abs(ref).max())
    if g == 1:
        assert np.array_equal(y, oracle.conv2d(x, w, b, s, p))
    if g == c == o:
        assert np.array_equal(y, oracle.dwconv2d(x, w, b, s, p))


@pytest.mark.parametrize("case", [(1, 7, 1, 0, 3), (7, 1, 1, 3, 0), (1, 3, 1, 0, 1), (3, 1, 2, 1, 0), (3, 3, 1, 1, 1), (5, 2, 2, 2, 0), (2, 4, 1, 1, 2)])
def test_rectangular_conv_vs_bruteforce_and_library(case, rng):
    """kh x kw kernels with separate paddings: against an explicit im2col x matmul written here, against a
    library routine in fp64, and (square case) bit for bit against the square convolution; a 1 x kw kernel
    applied to a transposed image equals the kw x 1 kernel's result transposed."""
    import torch.nn.functional as F
    kh, kw, s, ph, pw = case
    x = rng.standard_normal((2, 4, 10, 9)).astype(np.float32)
    w = rng.standard_normal((5, 4, kh, kw)).astype(np.float32)
    b = rng.standard_normal(5).astype(np.float32)
    y = oracle.conv2d_rect(x, w, b, s, ph, pw)
    xp = np.pad(x.astype(np.float64), ((0, 0), (0, 0), (ph, ph), (pw, pw)))
    ho, wo = (10 + 2 * ph - kh) // s + 1, (9 + 2 * pw - kw) // s + 1
    cols = np.empty((2, ho, wo, 4 * kh * kw))
    for i in range(ho):
        for j in range(wo):
            cols[:, i, j] = xp[:, :, i * s:i * s + kh, j * s:j * s + kw].reshape(2, -1)
    ref = (cols @ w.reshape(5, -1).astype(np.float64).T + b).transpose(0, 3, 1, 2)
    assert y.shape == ref.shape and np.abs(y - ref).max() < 1e-4
    lib = F.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(), torch.from_numpy(b).double(), s, (ph, pw)).numpy()
    assert np.abs(y - lib).max() < 1e-4
    if kh == kw and ph == pw:
        assert np.array_equal(y, oracle.conv2d(x, w, b, s, ph))
    yt = oracle.conv2d_rect(np.ascontiguousarray(x.transpose(0, 1, 3, 2)), np.ascontiguousarray(w.transpose(0, 1, 3, 2)), b, s, pw, ph)
    assert np.allclose(yt.transpose(0, 1, 3, 2), y, rtol=0, atol=1e-5)


def test_maxpool_ceil_mode_and_concat(rng):
    """Rounding the pooled size up lets windows hang over the far edge (those taps are never candidates) but
    never adds a window that starts past the input; the ramp's closed form and a library routine pin it.
    Concatenation is plane order: a's channels, then b's."""
    import torch.nn.functional as F
    x = np.arange(7 * 7, dtype=np.float32).reshape(1, 1, 7, 7)
    y = oracle.maxpool2d(x, 3, 2, 0, ceil=True)          # floor gives 3x3, ceil also 3x3: (7-3)/2 is whole
    assert y.shape == (1, 1, 3, 3) and np.array_equal(y, oracle.maxpool2d(x, 3, 2, 0))
    x = np.arange(8 * 8, dtype=np.float32).reshape(1, 1, 8, 8)
    y = oracle.maxpool2d(x, 3, 2, 0, ceil=True)          # floor 3x3, ceil 4x4: the last window holds rows/cols 6..7 only
    assert y.shape == (1, 1, 4, 4)
    want = np.array([[min(2 * i + 2, 7) * 8 + min(2 * j + 2, 7) for j in range(4)] for i in range(4)], dtype=np.float32)
    assert np.array_equal(y[0, 0], want)
    assert oracle.maxpool2d(np.zeros((1, 1, 5, 5), np.float32), 2, 2, 1, ceil=True).shape == (1, 1, 3, 3)  # not 4: window 3 would start in the padding past the input
    for (h, w, k, s, p) in [(13, 13, 3, 2, 0), (55, 57, 3, 2, 0), (7, 9, 3, 2, 1), (14, 14, 3, 1, 1), (27, 28, 3, 2, 0), (6, 6, 3, 2, 0), (5, 8, 2, 2, 0)]:
        x = -np.abs(rng.standard_normal((2, 3, h, w))).astype(np.float32)   # all negative: a zero from padding or overhang would win
        y = oracle.maxpool2d(x, k, s, p, ceil=True)
        ref = F.max_pool2d(torch.from_numpy(x), k, s, p, ceil_mode=True).numpy()
        assert y.shape == ref.shape and np.array_equal(y, ref)
    a = rng.standard_normal((2, 3, 4, 5)).astype(np.float32)
    b = rng.standard_normal((2, 2, 4, 5)).astype(np.float32)
    y = oracle.concat(a, b)
    assert y.shape == (2, 5, 4, 5) and np.array_equal(y[:, :3], a) and np.array_equal(y[:, 3:], b)
    assert np.array_equal(oracle.concat(a, a[:, :0]), a)


def test_avgpool_closed_forms_and_library(rng):
    """Window average: a constant stays the constant without padding and shrinks where the window hangs into
    zero padding (divisor is the full window area); a window covering the image is the global average; a
    library routine agrees."""
    import torch.nn.functional as F
    x = np.full((1, 2, 6, 6), 3.0, np.float32)
    assert np.array_equal(oracle.avgpool2d(x, 2, 2, 0), np.full((1, 2, 3, 3), 3.0, np.float32))
    y = oracle.avgpool2d(x, 3, 1, 1)
    assert y[0, 0, 0, 0] == np.float32(3.0 * 4 / 9) and y[0, 0, 0, 2] == np.float32(3.0 * 6 / 9) and y[0, 0, 2, 2] == 3.0
    ramp = np.arange(4 * 4, dtype=np.float32).reshape(1, 1, 4, 4)
    assert np.array_equal(oracle.avgpool2d(ramp, 2, 2, 0)[0, 0], np.array([[2.5, 4.5], [10.5, 12.5]], np.float32))
    x = rng.standard_normal((2, 3, 7, 7)).astype(np.float32)
    assert np.allclose(oracle.avgpool2d(x, 7, 1, 0).reshape(2, 3), oracle.global_avgpool(x), rtol=0, atol=1e-6)
    for (h, w, k, s, p) in [(8, 8, 2, 2, 0), (7, 9, 3, 1, 1), (14, 15, 3, 2, 1), (9, 6, 2, 2, 0), (5, 5, 5, 1, 2)]:
        x = rng.standard_normal((2, 3, h, w)).astype(np.float32)
        ref = F.avg_pool2d(torch.from_numpy(x).double(), k, s, p).numpy()
        y = oracle.avgpool2d(x, k, s, p)
        assert y.shape == ref.shape and np.abs(y - ref).max() < 1e-6


def test_global_avgpool_closed_forms():
    h, w = 7, 7
    ramp = np.arange(h * w, dtype=np.float32).reshape(1, 1, h, w)
    assert oracle.global_avgpool(ramp)[0, 0] == (h * w - 1) / 2
    const = np.full((2, 3, 4, 5), 2.5, dtype=np.float32)
    assert np.all(oracle.global_avgpool(const) == 2.5)
    x = np.zeros((1, 2, 3, 3), np.float32)
    x[0, 1] = 9.0  # channel separation
    assert np.array_equal(oracle.global_avgpool(x), np.array([[0.0, 9.0]], np.float32))


def test_fc_equals_matmul_and_1x1_and_7x7_valid_conv(rng):
    x = rng.standard_normal((3, 20)).astype(np.float32)
    w = rng.standard_normal((6, 20)).astype(np.float32)
    b = rng.standard_normal(6).astype(np.float32)
    y = oracle.fc(x, w, b)
    ref = x.astype(np.float64) @ w.astype(np.float64).T + b
    assert np.abs(y - ref).max() < 1e-5
    # non-square W catches a transposed operand; now FC == 1x1 conv on a 1x1 image
    y1 = oracle.conv2d(x.reshape(3, 20, 1, 1), w.reshape(6, 20, 1, 1), b, 1, 0).reshape(3, 6)
    assert np.abs(y - y1).max() < 1e-5
    # FC on a flattened C,H,W tensor == valid 7x7 conv down to 1x1
    xc = rng.standard_normal((2, 3, 7, 7)).astype(np.float32)
    wc = rng.standard_normal((4, 3, 7, 7)).astype(np.float32)
    bc = rng.standard_normal(4).astype(np.float32)
    yfc = oracle.fc(xc.reshape(2, -1), wc.reshape(4, -1), bc)
    ycv = oracle.conv2d(xc, wc, bc, 1, 0).reshape(2, 4)
    assert np.abs(yfc - ycv).max() < 1e-4


def test_softmax_closed_forms(rng):
    k = 10
    p = oracle.softmax(np.full((2, k), 3.0, dtype=np.float32))
    assert np.allclose(p, 1.0 / k, rtol=1e-6)
    z = rng.standard_normal((4, k)).astype(np.float32) * 5
    p = oracle.softmax(z)
    assert np.allclose(p.sum(axis=1), 1.0, atol=1e-6)
    assert np.allclose(oracle.softmax(z + 100.0), p, atol=1e-6)  # shift invariance
    # two-class closed form: softmax([a, 0]) = sigmoid(a)
    a = np.array([[2.0, 0.0], [-1.0, 0.0]], dtype=np.float32)
    sig = 1.0 / (1.0 + np.exp(-a[:, 0].astype(np.float64)))
    assert np.allclose(oracle.softmax(a)[:, 0], sig, atol=1e-6)
    big = np.array([[1000.0, 0.0, -1000.0]], dtype=np.float32)  # no overflow
    assert np.allclose(oracle.softmax(big), [[1.0, 0.0, 0.0]])


def test_activations_and_top1():
    v = np.array([-1.0, 0.0, 0.5, 6.0, 7.0], dtype=np.float32)
    assert np.array_equal(oracle.activate(v, "relu"), [0, 0, 0.5, 6, 7])
    assert np.array_equal(oracle.activate(v, "relu6"), [0, 0, 0.5, 6, 6])
    assert np.array_equal(oracle.activate(v, "none"), v)
    z = np.array([[1, 5, 5, 2], [9, 1, 9, 9]], dtype=np.float32)
    assert list(oracle.top1(z)) == [1, 0]  # lowest index on ties


def test_smooth_activations_and_channel_scale(rng):
    """Hard sigmoid is 0 below -3, 1 above 3 and (v+3)/6 between; hard swish is v times it; the logistic
    sigmoid satisfies s(0) = 1/2 and s(v) + s(-v) = 1, SiLU is v times it; a library routine agrees on a grid.
    The channel gate multiplies every pixel of plane (n, c) by g[n, c]."""
    import torch.nn.functional as F
    v = np.array([-7.0, -3.0, -1.5, 0.0, 1.5, 3.0, 7.0], np.float32)
    assert np.array_equal(oracle.activate(v.copy(), "hardsigmoid"), np.array([0, 0, 0.25, 0.5, 0.75, 1, 1], np.float32))
    assert np.array_equal(oracle.activate(v.copy(), "hardswish"), np.array([0, 0, -0.375, 0, 1.125, 3, 7], np.float32))
    s = oracle.activate(v.copy(), "sigmoid")
    assert s[3] == 0.5 and np.allclose(s + s[::-1], 1.0, atol=1e-7) and np.all(np.diff(s) > 0)
    assert np.allclose(oracle.activate(v.copy(), "silu"), v * s, atol=1e-7)
    grid = np.linspace(-9, 9, 721).astype(np.float32)
    for name, fn in (("hardswish", F.hardswish), ("hardsigmoid", F.hardsigmoid), ("silu", F.silu), ("sigmoid", torch.sigmoid)):
        ref = fn(torch.from_numpy(grid).double()).numpy()
        assert np.abs(oracle.activate(grid.copy(), name) - ref).max() < 1e-6
    x = rng.standard_normal((2, 3, 4, 5)).astype(np.float32)
    g = rng.standard_normal((2, 3)).astype(np.float32)
    assert np.array_equal(oracle.channel_scale(x, g), x * g[:, :, None, None])


def test_channel_slice_and_shuffle(rng):
    """A slice is a range of planes; a shuffle in G groups transposes the G x (C/G) channel matrix: with the
    channel index stored in the values it sends channel g*(C/G)+i to i*G+g, G = 1 and G = C are the identity,
    and shuffling by G then by C/G restores the input."""
    x = rng.standard_normal((2, 12, 3, 4)).astype(np.float32)
    assert np.array_equal(oracle.channel_slice(x, 5, 4), x[:, 5:9])
    assert np.array_equal(oracle.channel_slice(x, 0, 12), x)
    idx = np.broadcast_to(np.arange(12, dtype=np.float32)[None, :, None, None], (1, 12, 2, 2)).copy()
    y = oracle.channel_shuffle(idx, 3)[0, :, 0, 0]
    assert np.array_equal(y, np.array([0, 4, 8, 1, 5, 9, 2, 6, 10, 3, 7, 11], np.float32))
    assert np.array_equal(oracle.channel_shuffle(x, 1), x) and np.array_equal(oracle.channel_shuffle(x, 12), x)
    assert np.array_equal(oracle.channel_shuffle(oracle.channel_shuffle(x, 3), 4), x)
    ref = torch.from_numpy(x).view(2, 2, 6, 3, 4).transpose(1, 2).reshape(2, 12, 3, 4).numpy()
    assert np.array_equal(oracle.channel_shuffle(x, 2), ref)


def test_bf16_rounding_is_nearest_even():
    # 1 + 2^-8 is exactly half-way between bf16 neighbours 1 and 1 + 2^-7: ties go to even (1.0)
    assert oracle.round_bf16(np.array([1.0 + 2.0 ** -8], np.float32))[0] == 1.0
    # 1 + 3*2^-8 is half-way between 1+2^-7 (odd) and 1+2^-6 (even mantissa) -> up
    assert oracle.round_bf16(np.array([1.0 + 3 * 2.0 ** -8], np.float32))[0] == 1.0 + 2.0 ** -6
    assert oracle.round_bf16(np.array([1.0 + 2.0 ** -8 + 2.0 ** -20], np.float32))[0] == 1.0 + 2.0 ** -7
    x = np.random.default_rng(3).standard_normal(10000).astype(np.float32) * 100
    r = oracle.round_bf16(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).float().numpy()  # library rounding
    assert np.array_equal(r, ref)
    assert np.all(np.abs(r - x) <= np.abs(x) * 2.0 ** -8)


def test_two_bf16_terms_carry_two_to_the_minus_eight_of_bf16_storage_error(rng):
    """Tolerance derivation for members that keep fp32 activations: an fp32 value entering a bf16 product as
    hi = bf16(x) plus lo = bf16(x - hi) is perturbed by at most 2^-8 of what rounding it to one bf16 value does,
    element by element and therefore in every weighted sum (the oracle's own rounding routine, a plain matmul)."""
    x = rng.standard_normal((64, 4096)).astype(np.float32) * np.exp(rng.standard_normal((64, 4096))).astype(np.float32)
    w = oracle.round_bf16(rng.standard_normal((4096, 32)).astype(np.float32))
    hi = oracle.round_bf16(x)
    lo = oracle.round_bf16((x - hi).astype(np.float32))
    one = np.abs(hi.astype(np.float64) - x)
    two = np.abs(hi.astype(np.float64) + lo - x)
    assert np.all(two <= 2.0 ** -8 * np.abs(x) * 2.0 ** -8 * 1.0000001)          # two terms: 2^-17 relative at worst ...
    assert np.all(one <= 2.0 ** -8 * np.abs(x))                                  # ... one term: 2^-9 at worst
    y = x.astype(np.float64) @ w
    e_one = np.linalg.norm(hi.astype(np.float64) @ w - y)
    e_two = np.linalg.norm((hi.astype(np.float64) + lo) @ w - y)
    assert 0 < e_two <= 2.0 ** -8 * e_one
