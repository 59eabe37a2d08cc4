"""Seeded random layer graphs over every operator of the model description (data only, no arithmetic).

The named families exercise each operator in a handful of shapes; these graphs put the operators into
arbitrary order with odd channel counts, non-square inputs, residuals and concatenations across distant
nodes, so that both executors are compared on combinations no published architecture contains.
"""
from __future__ import annotations

import random

from . import zoo

ACTS = [zoo.NONE, zoo.RELU, zoo.RELU, zoo.RELU6, zoo.HARDSWISH, zoo.HARDSIGMOID, zoo.SILU, zoo.SIGMOID]


def random_model(seed: int, dtype: str = "bf16", in_c=None, hw=None, max_nodes: int = 14, large: bool = False,
                 aligned: bool = False) -> zoo.Model:
    """large: fewer nodes on bigger tensors (40-90 pixels a side, 64-512 channels), the shapes that reach the
    large convolution tiles.  aligned: channel counts mostly in multiples of 8 and, mixed into the random operators,
    the building blocks of the concatenating families (a dense layer: per-channel affine, 1x1, 3x3, concatenate;
    an Inception-style module with a pooling branch; a slice / branch / concatenate unit, often shuffled), so that
    concatenations whose sources can be stored in place and affine nodes a convolution can absorb occur next to
    ones that cannot.  The other modes draw exactly the graphs they always drew."""
    r = random.Random(seed)
    in_c = in_c or r.choice([1, 3, 3, 4, 8])
    lo, hi = (40, 90) if large else (9, 40)
    widths = [64, 64, 96, 128, 128, 192, 256, 320, 512] if large else [1, 3, 8, 10, 16, 24, 32, 40, 64, 72, 96, 130]
    if aligned:
        widths = [8, 12, 16, 20, 24, 32, 40, 58, 64, 64, 96, 116, 128]
    h, w = hw or ((lambda s: (s, s))(r.randint(lo, hi)) if r.random() < 0.6 else (r.randint(lo, hi), r.randint(lo, hi)))
    m = zoo.Model(f"rand{seed}", dtype, in_c, h, w)
    dims = {}   # node -> (c, h, w)

    def shape(node):
        return (in_c, h, w) if node == zoo.MODEL_INPUT else dims[node]

    def put(op, inp, out, **kw):
        i = m.add(op, inp, **kw)
        dims[i] = out
        return i

    cur = zoo.MODEL_INPUT
    for _ in range(r.randint(4 if large else 2, max_nodes)):
        c, hh, ww = shape(cur)
        act = r.choice(ACTS)
        what = r.random()
        if aligned and cur != zoo.MODEL_INPUT and r.random() < 0.4:
            block = r.randrange(3)
            if block == 0:     # dense layer
                g = r.choice([8, 16, 32])
                a = put(zoo.DWCONV, cur, (c, hh, ww), cin=c, cout=c, k=1, stride=1, pad=0, act=r.choice([zoo.RELU, zoo.RELU, zoo.NONE, zoo.RELU6, zoo.SILU]))
                a = put(zoo.CONV, a, (4 * g, hh, ww), cin=c, cout=4 * g, k=1, stride=1, pad=0, act=zoo.RELU)
                a = put(zoo.CONV, a, (g, hh, ww), cin=4 * g, cout=g, k=3, stride=1, pad=1, act=zoo.NONE)
                cur = put(zoo.CONCAT, cur, (c + g, hh, ww), residual=a)
            elif block == 1:   # module with a pooling branch
                c1, c2 = r.choice(widths), r.choice(widths)
                b1 = put(zoo.CONV, cur, (c1, hh, ww), cin=c, cout=c1, k=1, stride=1, pad=0, act=act)
                b2 = put(zoo.CONV, cur, (c2, hh, ww), cin=c, cout=c2, k=3, stride=1, pad=1, act=zoo.RELU)
                b3 = put(r.choice([zoo.MAXPOOL, zoo.AVGPOOL]), cur, (c, hh, ww), k=3, stride=1, pad=1)
                j = put(zoo.CONCAT, b1, (c1 + c2, hh, ww), residual=b2)
                cur = put(zoo.CONCAT, j, (c1 + c2 + c, hh, ww), residual=b3)
            elif c % 2 == 0 and c >= 4:   # kept half, worked half
                half = c // 2
                a = put(zoo.SLICE, cur, (half, hh, ww), first=0, cout=half)
                b = put(zoo.SLICE, cur, (half, hh, ww), first=half, cout=half)
                b = put(zoo.CONV, b, (half, hh, ww), cin=half, cout=half, k=1, stride=1, pad=0, act=zoo.RELU)
                cur = put(zoo.CONCAT, a, (c, hh, ww), residual=b)
                if r.random() < 0.6:   # ... and the two halves shuffled together, as a ShuffleNet unit ends
                    cur = put(zoo.SHUFFLE, cur, (c, hh, ww), groups=2)
            continue
        if large and what >= 0.42 and r.random() < 0.5:
            what = 0.0   # mostly dense convolutions
        if cur == zoo.MODEL_INPUT and what >= 0.64:
            what = 0.0   # the operators below do not take the model input directly
        if what < 0.42:
            k = r.choice([1, 1, 3, 3, 3, 5, 7]); kw = 0
            if r.random() < 0.15:
                k, kw = r.choice([(1, 3), (1, 7), (3, 1), (7, 1)])
            stride = 2 if r.random() < 0.25 else 1
            pad = max(k, kw) // 2 if r.random() < 0.7 else 0
            kww = kw or k
            ph, pw = (pad, pad) if kww == k else (pad if k > 1 else 0, pad if kww > 1 else 0)
            if hh + 2 * ph < k or ww + 2 * pw < kww:
                continue
            cout, groups = r.choice(widths), 1
            if not kw and r.random() < 0.2:
                g = r.choice([2, 4, 8])
                if c % g == 0:
                    groups, cout = g, g * r.randint(1, 12) * (4 if large else 1)
            out = (cout, (hh + 2 * ph - k) // stride + 1, (ww + 2 * pw - kww) // stride + 1)
            res = zoo.NO_RESIDUAL
            if r.random() < 0.4:
                same = [j for j in dims if dims[j] == out]
                if same:
                    res = r.choice(same)
            cur = put(zoo.CONV, cur, out, cin=c, cout=cout, k=k, kw=kw, stride=stride, pad=pad, act=act, residual=res, groups=groups)
        elif what < 0.52:
            k = r.choice([1, 1, 3, 5] if aligned else [3, 3, 5]); stride = 2 if r.random() < 0.3 else 1
            out = (c, (hh + 2 * (k // 2) - k) // stride + 1, (ww + 2 * (k // 2) - k) // stride + 1)
            cur = put(zoo.DWCONV, cur, out, cin=c, cout=c, k=k, stride=stride, pad=k // 2, act=act)
        elif what < 0.64:
            avg = r.random() < 0.4
            k = r.choice([2, 3]); stride = r.choice([1, 2]); pad = (k - 1) // 2 if r.random() < 0.5 else 0
            ceil = (not avg) and r.random() < 0.4
            if hh + 2 * pad < k or ww + 2 * pad < k:
                continue

            def pooled(n):
                if not ceil:
                    return (n + 2 * pad - k) // stride + 1
                o = -((n + 2 * pad - k) // -stride) + 1
                return o - 1 if (o - 1) * stride >= n + pad else o
            cur = put(zoo.AVGPOOL if avg else zoo.MAXPOOL, cur, (c, pooled(hh), pooled(ww)), k=k, stride=stride, pad=pad, ceil=ceil)
        elif what < 0.73:
            same = [j for j in dims if j != cur and dims[j][1:] == (hh, ww)]
            if not same:
                continue
            other = r.choice(same)
            cur = put(zoo.CONCAT, cur, (c + dims[other][0], hh, ww), residual=other)
        elif what < 0.82:   # squeeze-and-excitation gate
            sq = put(zoo.GAP, cur, (c, 1, 1))
            mid = r.randint(1, 16)
            f1 = put(zoo.CONV, sq, (mid, 1, 1), cin=c, cout=mid, k=1, act=zoo.RELU)
            f2 = put(zoo.CONV, f1, (c, 1, 1), cin=mid, cout=c, k=1, act=r.choice([zoo.SIGMOID, zoo.HARDSIGMOID]))
            cur = put(zoo.MUL, cur, (c, hh, ww), residual=f2)
        elif what < 0.90:
            if c < 2:
                continue
            first = r.randrange(c - 1); count = r.randint(1, c - first)
            cur = put(zoo.SLICE, cur, (count, hh, ww), first=first, cout=count)
        else:
            g = r.choice([2, 3, 4])
            if c % g:
                continue
            cur = put(zoo.SHUFFLE, cur, (c, hh, ww), groups=g)
    if cur == zoo.MODEL_INPUT:
        cur = put(zoo.CONV, cur, (8, h, w), cin=in_c, cout=8, k=1, act=zoo.RELU)
    if r.random() < 0.8:   # classifier head
        c, hh, ww = shape(cur)
        if r.random() < 0.7:
            cur = put(zoo.GAP, cur, (c, 1, 1)); hh = ww = 1
        classes = r.choice([1, 10, 37, 1000])
        cur = put(zoo.FC, cur, (classes, 1, 1), cin=c * hh * ww, cout=classes, act=zoo.RELU if r.random() < 0.2 else zoo.NONE)
        if r.random() < 0.3:
            cur = put(zoo.SOFTMAX, cur, (classes, 1, 1))
    m.shapes()
    for i, L in enumerate(m.layers):   # the bookkeeping above and the description's own shape inference agree
        assert (L.cout, L.out_h, L.out_w) == dims[i], (seed, i, L, dims[i])
    return m
