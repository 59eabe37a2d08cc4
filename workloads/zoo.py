"""Layer-graph descriptions of the member models (data only, no arithmetic).

A model is a list of nodes in topological order.  Each node names its operator,
the node that feeds it (-1 = the model input), an optional residual node that
is added before the activation, and the operator's integer hyper-parameters.
This is the per-model graph (nodes u_i, edges {u_i,u_j}, activations phi_i)
that the paper's Algorithm 1 unions into one DAG.

The first five families are the ones the benchmark configurations name: a tiny
CNN, ResNet-18 / ResNet-50 (BatchNorm folded into the preceding convolution, so
each convolution carries one bias per output channel), MobileNetV2 (width 1.0)
and VGG-16; the others are families of the paper's Table III that the same five
operators cover (AlexNet, VGG-11/13/19, ResNet-34/101/152, Wide ResNet-50-2 /
101-2, MnasNet 1.0).  Shapes follow the published architecture tables; the
bottleneck ResNets carry the stride on their 3x3 convolution.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List

# operator / activation names (strings on purpose: each executor maps them to
# its own enum, so the two sides share no numeric constants)
CONV, DWCONV, MAXPOOL, GAP, FC, SOFTMAX, CONCAT, AVGPOOL, MUL, SLICE, SHUFFLE = "conv", "dwconv", "maxpool", "gap", "fc", "softmax", "concat", "avgpool", "mul", "slice", "shuffle"
NONE, RELU, RELU6, HARDSWISH, HARDSIGMOID, SILU, SIGMOID = "none", "relu", "relu6", "hardswish", "hardsigmoid", "silu", "sigmoid"
NO_RESIDUAL = -2
MODEL_INPUT = -1


@dataclass
class Layer:
    op: str
    input: int
    cin: int = 0
    cout: int = 0
    k: int = 1
    stride: int = 1
    pad: int = 0
    act: str = NONE
    residual: int = NO_RESIDUAL   # node added before the activation; for a concat node: the second source
    ceil: bool = False            # pooling: output size rounds up (windows may hang over the bottom / right edge)
    groups: int = 1               # conv: input and output channels are cut into this many independent groups; shuffle: groups
    first: int = 0                # slice: first channel taken (cout channels from there)
    kw: int = 0                   # conv: kernel width when it differs from the height k (0 = square); `pad` then
                                  # applies only along a dimension the kernel extends over (size > 1)
    bias: bool = True             # False: the layer has no bias in the architecture (its stored bias is all zero)
    bn: bool = True               # conv / depthwise with a bias: the bias stands for a folded BatchNorm
    # filled by shapes(): logical input / output spatial sizes
    in_h: int = 0
    in_w: int = 0
    out_h: int = 0
    out_w: int = 0
    # filled by gen.make_blob(): byte offsets into the canonical weight blob
    w_off: int = 0
    b_off: int = 0


@dataclass
class Model:
    name: str
    dtype: str  # "f32" | "bf16"
    in_c: int
    in_h: int
    in_w: int
    layers: List[Layer] = field(default_factory=list)

    @property
    def output(self) -> int:
        return len(self.layers) - 1

    def add(self, op, inp, **kw) -> int:
        self.layers.append(Layer(op=op, input=inp, **kw))
        return len(self.layers) - 1

    # -- derived facts used by structural pins ------------------------------
    def shapes(self) -> "Model":
        """Fill in per-node logical shapes (floor output size, except pooling nodes that ask for ceil)."""
        def pooled(n, L):
            if not L.ceil:
                return (n + 2 * L.pad - L.k) // L.stride + 1
            out = -((n + 2 * L.pad - L.k) // -L.stride) + 1
            if (out - 1) * L.stride >= n + L.pad:   # the last window must start inside the input or its left padding
                out -= 1
            return out
        dims = {}
        for i, L in enumerate(self.layers):
            c, h, w = (self.in_c, self.in_h, self.in_w) if L.input == MODEL_INPUT else dims[L.input]
            L.in_h, L.in_w = h, w
            if L.op in (CONV, DWCONV):
                kw = L.kw or L.k
                ph, pw = (L.pad, L.pad) if kw == L.k else (L.pad if L.k > 1 else 0, L.pad if kw > 1 else 0)
                ho = (h + 2 * ph - L.k) // L.stride + 1
                wo = (w + 2 * pw - kw) // L.stride + 1
                dims[i] = (L.cout, ho, wo)
            elif L.op in (MAXPOOL, AVGPOOL):
                assert not (L.op == AVGPOOL and L.ceil)
                L.cin = L.cout = c
                dims[i] = (c, pooled(h, L), pooled(w, L))
            elif L.op == SLICE:
                assert 0 <= L.first and L.first + L.cout <= c, (self.name, i)
                L.cin = c
                dims[i] = (L.cout, h, w)
            elif L.op == SHUFFLE:
                assert c % L.groups == 0, (self.name, i)
                L.cin = L.cout = c
                dims[i] = (c, h, w)
            elif L.op == MUL:      # `input` scaled per (image, channel) by the 1x1 tensor `residual`
                c2, h2, w2 = dims[L.residual]
                assert (c2, h2, w2) == (c, 1, 1), (self.name, i)
                L.cin = L.cout = c
                dims[i] = (c, h, w)
            elif L.op == CONCAT:   # channels of `input`, then channels of `residual`
                c2, h2, w2 = dims[L.residual]
                assert (h2, w2) == (h, w), (self.name, i)
                L.cin, L.cout = c, c + c2
                dims[i] = (c + c2, h, w)
            elif L.op == GAP:
                L.cin = L.cout = c
                dims[i] = (c, 1, 1)
            elif L.op == FC:
                assert L.cin == c * h * w, (self.name, i, L.cin, c, h, w)
                dims[i] = (L.cout, 1, 1)
            elif L.op == SOFTMAX:
                L.cin = L.cout = c
                dims[i] = (c, 1, 1)
            else:
                raise ValueError(L.op)
            L.out_h, L.out_w = dims[i][1], dims[i][2]
        return self

    def n_params(self) -> int:
        n = 0
        for L in self.layers:
            b = L.cout if L.bias else 0
            if L.op == CONV:
                n += L.cout * (L.cin // L.groups) * L.k * (L.kw or L.k) + b
            elif L.op == DWCONV:
                n += L.cout * L.k * L.k + b
            elif L.op == FC:
                n += L.cout * L.cin + b
        return n

    def macs(self) -> int:
        """Multiply-accumulates per image of conv / depthwise / FC nodes."""
        n = 0
        for L in self.layers:
            if L.op == CONV:
                n += L.out_h * L.out_w * L.cout * (L.cin // L.groups) * L.k * (L.kw or L.k)
            elif L.op == DWCONV:
                n += L.out_h * L.out_w * L.cout * L.k * L.k
            elif L.op == FC:
                n += L.cout * L.cin
        return n

    def levels(self) -> List[int]:
        """Depth of every node: 1 + max depth of its inputs (model input = 0)."""
        lv = []
        for L in self.layers:
            d = 0 if L.input == MODEL_INPUT else lv[L.input]
            if L.residual >= 0:
                d = max(d, lv[L.residual])
            lv.append(d + 1)
        return lv


def tiny_cnn(dtype: str = "f32", softmax: bool = True) -> Model:
    m = Model("tiny", dtype, 3, 32, 32)
    a = m.add(CONV, MODEL_INPUT, cin=3, cout=16, k=3, stride=1, pad=1, act=RELU)
    a = m.add(MAXPOOL, a, k=2, stride=2, pad=0)
    a = m.add(CONV, a, cin=16, cout=32, k=3, stride=1, pad=1, act=RELU)
    a = m.add(GAP, a)
    a = m.add(FC, a, cin=32, cout=10)
    if softmax:
        m.add(SOFTMAX, a)
    return m.shapes()


def _resnet_stem(m: Model) -> int:
    a = m.add(CONV, MODEL_INPUT, cin=3, cout=64, k=7, stride=2, pad=3, act=RELU)
    return m.add(MAXPOOL, a, k=3, stride=2, pad=1)


def _basic_resnet(name: str, reps, dtype: str, classes: int, hw: int) -> Model:
    """ResNet with two-convolution basic blocks (He et al. 2016, Table 1: 18 and 34 layers)."""
    m = Model(name, dtype, 3, hw, hw)
    x = _resnet_stem(m)
    cin = 64
    for stage, (width, n) in enumerate(zip((64, 128, 256, 512), reps)):
        for blk in range(n):
            stride = 2 if (stage > 0 and blk == 0) else 1
            a = m.add(CONV, x, cin=cin, cout=width, k=3, stride=stride, pad=1, act=RELU)
            if stride != 1 or cin != width:
                skip = m.add(CONV, x, cin=cin, cout=width, k=1, stride=stride, pad=0, act=NONE)
            else:
                skip = x
            x = m.add(CONV, a, cin=width, cout=width, k=3, stride=1, pad=1, act=RELU, residual=skip)
            cin = width
    x = m.add(GAP, x)
    m.add(FC, x, cin=512, cout=classes)
    return m.shapes()


def _bottleneck_resnet(name: str, reps, inner: int, dtype: str, classes: int, hw: int, groups: int = 1) -> Model:
    """ResNet with 1x1 / 3x3 / 1x1 bottleneck blocks (50, 101, 152 layers); `inner` scales the width of
    the two inner convolutions (2 for the wide variants of Zagoruyko & Komodakis 2016; 2 with 32 groups in
    the 3x3 is ResNeXt 32x4d, Xie et al. 2017).  Stride on the 3x3."""
    m = Model(name, dtype, 3, hw, hw)
    x = _resnet_stem(m)
    cin = 64
    for stage, (width, n) in enumerate(zip((64, 128, 256, 512), reps)):
        mid = width * inner
        for blk in range(n):
            stride = 2 if (stage > 0 and blk == 0) else 1
            a = m.add(CONV, x, cin=cin, cout=mid, k=1, stride=1, pad=0, act=RELU)
            if blk == 0:
                skip = m.add(CONV, x, cin=cin, cout=4 * width, k=1, stride=stride, pad=0, act=NONE)
            else:
                skip = x
            a = m.add(CONV, a, cin=mid, cout=mid, k=3, stride=stride, pad=1, act=RELU, groups=groups)
            x = m.add(CONV, a, cin=mid, cout=4 * width, k=1, stride=1, pad=0, act=RELU, residual=skip)
            cin = 4 * width
    x = m.add(GAP, x)
    m.add(FC, x, cin=2048, cout=classes)
    return m.shapes()


def resnet18(dtype: str = "bf16", classes: int = 1000, hw: int = 224) -> Model:
    return _basic_resnet("resnet18", (2, 2, 2, 2), dtype, classes, hw)


def resnet34(dtype: str = "bf16", classes: int = 1000, hw: int = 224) -> Model:
    return _basic_resnet("resnet34", (3, 4, 6, 3), dtype, classes, hw)


def resnet50(dtype: str = "bf16", classes: int = 1000, hw: int = 224) -> Model:
    return _bottleneck_resnet("resnet50", (3, 4, 6, 3), 1, dtype, classes, hw)


def resnet101(dtype: str = "bf16", classes: int = 1000, hw: int = 224) -> Model:
    return _bottleneck_resnet("resnet101", (3, 4, 23, 3), 1, dtype, classes, hw)


def resnet152(dtype: str = "bf16", classes: int = 1000, hw: int = 224) -> Model:
    return _bottleneck_resnet("resnet152", (3, 8, 36, 3), 1, dtype, classes, hw)


def wide_resnet50_2(dtype: str = "bf16", classes: int = 1000, hw: int = 224) -> Model:
    return _bottleneck_resnet("wide_resnet50_2", (3, 4, 6, 3), 2, dtype, classes, hw)


def resnext50_32x4d(dtype: str = "bf16", classes: int = 1000, hw: int = 224) -> Model:
    return _bottleneck_resnet("resnext50_32x4d", (3, 4, 6, 3), 2, dtype, classes, hw, groups=32)


def resnext101_32x8d(dtype: str = "bf16", classes: int = 1000, hw: int = 224) -> Model:
    return _bottleneck_resnet("resnext101_32x8d", (3, 4, 23, 3), 4, dtype, classes, hw, groups=32)


def wide_resnet101_2(dtype: str = "bf16", classes: int = 1000, hw: int = 224) -> Model:
    return _bottleneck_resnet("wide_resnet101_2", (3, 4, 23, 3), 2, dtype, classes, hw)


def mobilenetv2(dtype: str = "bf16", classes: int = 1000, hw: int = 224) -> Model:
    m = Model("mobilenetv2", dtype, 3, hw, hw)
    x = m.add(CONV, MODEL_INPUT, cin=3, cout=32, k=3, stride=2, pad=1, act=RELU6)
    cin = 32
    for t, c, n, s in ((1, 16, 1, 1), (6, 24, 2, 2), (6, 32, 3, 2), (6, 64, 4, 2),
                       (6, 96, 3, 1), (6, 160, 3, 2), (6, 320, 1, 1)):
        for rep in range(n):
            stride = s if rep == 0 else 1
            hidden = cin * t
            a = x
            if t != 1:
                a = m.add(CONV, a, cin=cin, cout=hidden, k=1, stride=1, pad=0, act=RELU6)
            a = m.add(DWCONV, a, cin=hidden, cout=hidden, k=3, stride=stride, pad=1, act=RELU6)
            skip = x if (stride == 1 and cin == c) else NO_RESIDUAL
            x = m.add(CONV, a, cin=hidden, cout=c, k=1, stride=1, pad=0, act=NONE, residual=skip)
            cin = c
    x = m.add(CONV, x, cin=320, cout=1280, k=1, stride=1, pad=0, act=RELU6)
    x = m.add(GAP, x)
    m.add(FC, x, cin=1280, cout=classes)
    return m.shapes()


_VGG = {  # Simonyan & Zisserman 2015, Table 1: configurations A, B, D, E
    "vgg11": (64, "M", 128, "M", 256, 256, "M", 512, 512, "M", 512, 512, "M"),
    "vgg13": (64, 64, "M", 128, 128, "M", 256, 256, "M", 512, 512, "M", 512, 512, "M"),
    "vgg16": (64, 64, "M", 128, 128, "M", 256, 256, 256, "M", 512, 512, 512, "M", 512, 512, 512, "M"),
    "vgg19": (64, 64, "M", 128, 128, "M", 256, 256, 256, 256, "M", 512, 512, 512, 512, "M", 512, 512, 512, 512, "M"),
}


def _vgg(name: str, dtype: str, classes: int, hw: int) -> Model:
    m = Model(name, dtype, 3, hw, hw)
    x, cin, side = MODEL_INPUT, 3, hw
    for v in _VGG[name]:
        if v == "M":
            x = m.add(MAXPOOL, x, k=2, stride=2, pad=0)
            side //= 2
        else:
            x = m.add(CONV, x, cin=cin, cout=v, k=3, stride=1, pad=1, act=RELU)
            cin = v
    x = m.add(FC, x, cin=512 * side * side, cout=4096, act=RELU)
    x = m.add(FC, x, cin=4096, cout=4096, act=RELU)
    m.add(FC, x, cin=4096, cout=classes)
    return m.shapes()


def vgg11(dtype: str = "bf16", classes: int = 1000, hw: int = 224) -> Model:
    return _vgg("vgg11", dtype, classes, hw)


def vgg13(dtype: str = "bf16", classes: int = 1000, hw: int = 224) -> Model:
    return _vgg("vgg13", dtype, classes, hw)


def vgg16(dtype: str = "bf16", classes: int = 1000, hw: int = 224) -> Model:
    return _vgg("vgg16", dtype, classes, hw)


def vgg19(dtype: str = "bf16", classes: int = 1000, hw: int = 224) -> Model:
    return _vgg("vgg19", dtype, classes, hw)


def alexnet(dtype: str = "bf16", classes: int = 1000, hw: int = 224) -> Model:
    """The single-tower AlexNet (Krizhevsky 2014): 11x11/4, 5x5 and three 3x3 convolutions, 3x3/2 max
    pooling after the first, second and fifth, three fully connected layers (6x6x256 inputs at 224)."""
    m = Model("alexnet", dtype, 3, hw, hw)
    side = (hw + 2 * 2 - 11) // 4 + 1
    x = m.add(CONV, MODEL_INPUT, cin=3, cout=64, k=11, stride=4, pad=2, act=RELU)
    x = m.add(MAXPOOL, x, k=3, stride=2, pad=0)
    side = (side - 3) // 2 + 1
    x = m.add(CONV, x, cin=64, cout=192, k=5, stride=1, pad=2, act=RELU)
    x = m.add(MAXPOOL, x, k=3, stride=2, pad=0)
    side = (side - 3) // 2 + 1
    x = m.add(CONV, x, cin=192, cout=384, k=3, stride=1, pad=1, act=RELU)
    x = m.add(CONV, x, cin=384, cout=256, k=3, stride=1, pad=1, act=RELU)
    x = m.add(CONV, x, cin=256, cout=256, k=3, stride=1, pad=1, act=RELU)
    x = m.add(MAXPOOL, x, k=3, stride=2, pad=0)
    side = (side - 3) // 2 + 1
    x = m.add(FC, x, cin=256 * side * side, cout=4096, act=RELU)
    x = m.add(FC, x, cin=4096, cout=4096, act=RELU)
    m.add(FC, x, cin=4096, cout=classes)
    return m.shapes()


def mnasnet1_0(dtype: str = "bf16", classes: int = 1000, hw: int = 224) -> Model:
    """MnasNet-A1 without squeeze-excite at depth multiplier 1.0 (Tan et al. 2019, the B1 variant): a
    separable stem, then inverted residuals (expansion, kernel, stride, repeats, width) with ReLU."""
    m = Model("mnasnet1_0", dtype, 3, hw, hw)
    x = m.add(CONV, MODEL_INPUT, cin=3, cout=32, k=3, stride=2, pad=1, act=RELU)
    x = m.add(DWCONV, x, cin=32, cout=32, k=3, stride=1, pad=1, act=RELU)
    x = m.add(CONV, x, cin=32, cout=16, k=1, stride=1, pad=0, act=NONE)
    cin = 16
    for t, k, s, n, c in ((3, 3, 2, 3, 24), (3, 5, 2, 3, 40), (6, 5, 2, 3, 80), (6, 3, 1, 2, 96), (6, 5, 2, 4, 192), (6, 3, 1, 1, 320)):
        for rep in range(n):
            stride = s if rep == 0 else 1
            hidden = cin * t
            a = m.add(CONV, x, cin=cin, cout=hidden, k=1, stride=1, pad=0, act=RELU)
            a = m.add(DWCONV, a, cin=hidden, cout=hidden, k=k, stride=stride, pad=k // 2, act=RELU)
            skip = x if (stride == 1 and cin == c) else NO_RESIDUAL
            x = m.add(CONV, a, cin=hidden, cout=c, k=1, stride=1, pad=0, act=NONE, residual=skip)
            cin = c
    x = m.add(CONV, x, cin=320, cout=1280, k=1, stride=1, pad=0, act=RELU)
    x = m.add(GAP, x)
    m.add(FC, x, cin=1280, cout=classes)
    return m.shapes()


def squeezenet1_1(dtype: str = "bf16", classes: int = 1000, hw: int = 224) -> Model:
    """SqueezeNet 1.1 (Iandola et al. 2016, the lighter revision): fire modules = 1x1 squeeze, then 1x1 and
    3x3 expands side by side, concatenated; 3x3/2 max pooling with the size rounded up; a 1x1 classifier
    convolution followed by global average pooling (no fully connected layer, no BatchNorm)."""
    m = Model("squeezenet1_1", dtype, 3, hw, hw)
    x = m.add(CONV, MODEL_INPUT, cin=3, cout=64, k=3, stride=2, pad=0, act=RELU)
    x = m.add(MAXPOOL, x, k=3, stride=2, pad=0, ceil=True)
    cin = 64
    for idx, (sq, ex) in enumerate(((16, 64), (16, 64), (32, 128), (32, 128), (48, 192), (48, 192), (64, 256), (64, 256))):
        if idx in (2, 4):
            x = m.add(MAXPOOL, x, k=3, stride=2, pad=0, ceil=True)
        q = m.add(CONV, x, cin=cin, cout=sq, k=1, stride=1, pad=0, act=RELU)
        e1 = m.add(CONV, q, cin=sq, cout=ex, k=1, stride=1, pad=0, act=RELU)
        e3 = m.add(CONV, q, cin=sq, cout=ex, k=3, stride=1, pad=1, act=RELU)
        x = m.add(CONCAT, e1, residual=e3)
        cin = 2 * ex
    x = m.add(CONV, x, cin=512, cout=classes, k=1, stride=1, pad=0, act=RELU)
    m.add(GAP, x)
    return m.shapes()


def _divisible(v: float, d: int = 8) -> int:
    n = max(d, int(v + d / 2) // d * d)
    return n + d if n < 0.9 * v else n


def _mobilenetv3(name: str, cfg, last: int, head: int, dtype: str, classes: int, hw: int) -> Model:
    """MobileNetV3 (Howard et al. 2019, Tables 1 and 2): inverted residuals (kernel, expansion, width,
    squeeze-excite, activation, stride); the squeeze-excite gate is global average -> FC (ReLU) -> FC (hard
    sigmoid) with expansion/4 (rounded to 8) hidden units, applied per channel before the projection."""
    m = Model(name, dtype, 3, hw, hw)
    x = m.add(CONV, MODEL_INPUT, cin=3, cout=16, k=3, stride=2, pad=1, act=HARDSWISH)
    cin = 16
    for k, exp, c, se, act, stride in cfg:
        a = x
        if exp != cin:
            a = m.add(CONV, a, cin=cin, cout=exp, k=1, stride=1, pad=0, act=act)
        a = m.add(DWCONV, a, cin=exp, cout=exp, k=k, stride=stride, pad=k // 2, act=act)
        if se:
            sq = _divisible(exp // 4)
            g = m.add(GAP, a)
            g = m.add(FC, g, cin=exp, cout=sq, act=RELU)
            g = m.add(FC, g, cin=sq, cout=exp, act=HARDSIGMOID)
            a = m.add(MUL, a, residual=g)
        skip = x if (stride == 1 and cin == c) else NO_RESIDUAL
        x = m.add(CONV, a, cin=exp, cout=c, k=1, stride=1, pad=0, act=NONE, residual=skip)
        cin = c
    x = m.add(CONV, x, cin=cin, cout=last, k=1, stride=1, pad=0, act=HARDSWISH)
    x = m.add(GAP, x)
    x = m.add(FC, x, cin=last, cout=head, act=HARDSWISH)
    m.add(FC, x, cin=head, cout=classes)
    return m.shapes()


def mobilenet_v3_large(dtype: str = "bf16", classes: int = 1000, hw: int = 224) -> Model:
    R, H = RELU, HARDSWISH
    cfg = ((3, 16, 16, False, R, 1), (3, 64, 24, False, R, 2), (3, 72, 24, False, R, 1), (5, 72, 40, True, R, 2),
           (5, 120, 40, True, R, 1), (5, 120, 40, True, R, 1), (3, 240, 80, False, H, 2), (3, 200, 80, False, H, 1),
           (3, 184, 80, False, H, 1), (3, 184, 80, False, H, 1), (3, 480, 112, True, H, 1), (3, 672, 112, True, H, 1),
           (5, 672, 160, True, H, 2), (5, 960, 160, True, H, 1), (5, 960, 160, True, H, 1))
    return _mobilenetv3("mobilenet_v3_large", cfg, 960, 1280, dtype, classes, hw)


def mobilenet_v3_small(dtype: str = "bf16", classes: int = 1000, hw: int = 224) -> Model:
    R, H = RELU, HARDSWISH
    cfg = ((3, 16, 16, True, R, 2), (3, 72, 24, False, R, 2), (3, 88, 24, False, R, 1), (5, 96, 40, True, H, 2),
           (5, 240, 40, True, H, 1), (5, 240, 40, True, H, 1), (5, 120, 48, True, H, 1), (5, 144, 48, True, H, 1),
           (5, 288, 96, True, H, 2), (5, 576, 96, True, H, 1), (5, 576, 96, True, H, 1))
    return _mobilenetv3("mobilenet_v3_small", cfg, 576, 1024, dtype, classes, hw)


def _efficientnet_v2(name: str, stages, dtype: str, classes: int, hw: int) -> Model:
    """EfficientNetV2 (Tan & Le 2021, Table 4): fused blocks (3x3 expansion convolution, 1x1 projection) in
    the early stages, then depthwise blocks with a squeeze-excite gate whose hidden width is a quarter of
    the block's input width; SiLU throughout, a sigmoid on the gate.  stages: (fused, expansion, stride,
    width, repeats)."""
    m = Model(name, dtype, 3, hw, hw)
    cin = stages[0][3]
    x = m.add(CONV, MODEL_INPUT, cin=3, cout=cin, k=3, stride=2, pad=1, act=SILU)
    for fused, e, s0, c, n in stages:
        for rep in range(n):
            stride = s0 if rep == 0 else 1
            skip = x if (stride == 1 and cin == c) else NO_RESIDUAL
            if fused and e == 1:
                x = m.add(CONV, x, cin=cin, cout=c, k=3, stride=stride, pad=1, act=SILU, residual=skip)
            elif fused:
                a = m.add(CONV, x, cin=cin, cout=cin * e, k=3, stride=stride, pad=1, act=SILU)
                x = m.add(CONV, a, cin=cin * e, cout=c, k=1, stride=1, pad=0, act=NONE, residual=skip)
            else:
                a = m.add(CONV, x, cin=cin, cout=cin * e, k=1, stride=1, pad=0, act=SILU)
                a = m.add(DWCONV, a, cin=cin * e, cout=cin * e, k=3, stride=stride, pad=1, act=SILU)
                g = m.add(GAP, a)
                g = m.add(FC, g, cin=cin * e, cout=max(1, cin // 4), act=SILU)
                g = m.add(FC, g, cin=max(1, cin // 4), cout=cin * e, act=SIGMOID)
                a = m.add(MUL, a, residual=g)
                x = m.add(CONV, a, cin=cin * e, cout=c, k=1, stride=1, pad=0, act=NONE, residual=skip)
            cin = c
    x = m.add(CONV, x, cin=cin, cout=1280, k=1, stride=1, pad=0, act=SILU)
    x = m.add(GAP, x)
    m.add(FC, x, cin=1280, cout=classes)
    return m.shapes()


def efficientnet_v2_s(dtype: str = "bf16", classes: int = 1000, hw: int = 384) -> Model:
    return _efficientnet_v2("efficientnet_v2_s", ((True, 1, 1, 24, 2), (True, 4, 2, 48, 4), (True, 4, 2, 64, 4),
                            (False, 4, 2, 128, 6), (False, 6, 1, 160, 9), (False, 6, 2, 256, 15)), dtype, classes, hw)


def efficientnet_v2_m(dtype: str = "bf16", classes: int = 1000, hw: int = 480) -> Model:
    return _efficientnet_v2("efficientnet_v2_m", ((True, 1, 1, 24, 3), (True, 4, 2, 48, 5), (True, 4, 2, 80, 5), (False, 4, 2, 160, 7),
                            (False, 6, 1, 176, 14), (False, 6, 2, 304, 18), (False, 6, 1, 512, 5)), dtype, classes, hw)


def efficientnet_v2_l(dtype: str = "bf16", classes: int = 1000, hw: int = 480) -> Model:
    return _efficientnet_v2("efficientnet_v2_l", ((True, 1, 1, 32, 4), (True, 4, 2, 64, 7), (True, 4, 2, 96, 7), (False, 4, 2, 192, 10),
                            (False, 6, 1, 224, 19), (False, 6, 2, 384, 25), (False, 6, 1, 640, 7)), dtype, classes, hw)


def _shufflenet_v2(name: str, widths, dtype: str, classes: int, hw: int) -> Model:
    """ShuffleNet V2 (Ma et al. 2018, Table 5): a unit keeps half of its channels and sends the other half
    through 1x1 -> 3x3 depthwise (no activation) -> 1x1, concatenates and shuffles the channels in two groups;
    a down-sampling unit runs both halves from the whole input, the first through depthwise/2 -> 1x1."""
    m = Model(name, dtype, 3, hw, hw)
    x = m.add(CONV, MODEL_INPUT, cin=3, cout=24, k=3, stride=2, pad=1, act=RELU)
    x = m.add(MAXPOOL, x, k=3, stride=2, pad=1)
    cin = 24
    for c, reps in zip(widths[:3], (4, 8, 4)):
        half = c // 2
        for rep in range(reps):
            if rep == 0:
                a = m.add(DWCONV, x, cin=cin, cout=cin, k=3, stride=2, pad=1, act=NONE)
                a = m.add(CONV, a, cin=cin, cout=half, k=1, stride=1, pad=0, act=RELU)
                b = m.add(CONV, x, cin=cin, cout=half, k=1, stride=1, pad=0, act=RELU)
                b = m.add(DWCONV, b, cin=half, cout=half, k=3, stride=2, pad=1, act=NONE)
            else:
                a = m.add(SLICE, x, first=0, cout=half)
                b = m.add(SLICE, x, first=half, cout=half)
                b = m.add(CONV, b, cin=half, cout=half, k=1, stride=1, pad=0, act=RELU)
                b = m.add(DWCONV, b, cin=half, cout=half, k=3, stride=1, pad=1, act=NONE)
            b = m.add(CONV, b, cin=half, cout=half, k=1, stride=1, pad=0, act=RELU)
            x = m.add(CONCAT, a, residual=b)
            x = m.add(SHUFFLE, x, groups=2)
            cin = c
    x = m.add(CONV, x, cin=cin, cout=widths[3], k=1, stride=1, pad=0, act=RELU)
    x = m.add(GAP, x)
    m.add(FC, x, cin=widths[3], cout=classes)
    return m.shapes()


def shufflenet_v2_x1_0(dtype: str = "bf16", classes: int = 1000, hw: int = 224) -> Model:
    return _shufflenet_v2("shufflenet_v2_x1_0", (116, 232, 464, 1024), dtype, classes, hw)


def shufflenet_v2_x0_5(dtype: str = "bf16", classes: int = 1000, hw: int = 224) -> Model:
    return _shufflenet_v2("shufflenet_v2_x0_5", (48, 96, 192, 1024), dtype, classes, hw)


def inception_v3(dtype: str = "bf16", classes: int = 1000, hw: int = 299) -> Model:
    """Inception v3 (Szegedy et al. 2016) without the auxiliary head: factorised 5x5 -> two 3x3, n x n -> 1 x n
    and n x 1 pairs, average-pool branches, grid reductions that concatenate strided convolutions with a
    max pool."""
    m = Model("inception_v3", dtype, 3, hw, hw)

    def conv(x, cin, cout, k, stride=1, pad=0, kw=0):
        return m.add(CONV, x, cin=cin, cout=cout, k=k, kw=kw, stride=stride, pad=pad, act=RELU)

    def cat(parts):
        y, c = parts[0]
        for z, cz in parts[1:]:
            y = m.add(CONCAT, y, residual=z)
            c += cz
        return y, c

    def block_a(x, cin, pf):
        b1 = conv(x, cin, 64, 1)
        b2 = conv(conv(x, cin, 48, 1), 48, 64, 5, pad=2)
        b3 = conv(conv(conv(x, cin, 64, 1), 64, 96, 3, pad=1), 96, 96, 3, pad=1)
        b4 = conv(m.add(AVGPOOL, x, k=3, stride=1, pad=1), cin, pf, 1)
        return cat([(b1, 64), (b2, 64), (b3, 96), (b4, pf)])

    def block_b(x, cin):
        b1 = conv(x, cin, 384, 3, stride=2)
        b2 = conv(conv(conv(x, cin, 64, 1), 64, 96, 3, pad=1), 96, 96, 3, stride=2)
        b3 = m.add(MAXPOOL, x, k=3, stride=2, pad=0)
        return cat([(b1, 384), (b2, 96), (b3, cin)])

    def block_c(x, cin, c7):
        b1 = conv(x, cin, 192, 1)
        b2 = conv(conv(conv(x, cin, c7, 1), c7, c7, 1, kw=7, pad=3), c7, 192, 7, kw=1, pad=3)
        b3 = conv(x, cin, c7, 1)
        b3 = conv(b3, c7, c7, 7, kw=1, pad=3)
        b3 = conv(b3, c7, c7, 1, kw=7, pad=3)
        b3 = conv(b3, c7, c7, 7, kw=1, pad=3)
        b3 = conv(b3, c7, 192, 1, kw=7, pad=3)
        b4 = conv(m.add(AVGPOOL, x, k=3, stride=1, pad=1), cin, 192, 1)
        return cat([(b1, 192), (b2, 192), (b3, 192), (b4, 192)])

    def block_d(x, cin):
        b1 = conv(conv(x, cin, 192, 1), 192, 320, 3, stride=2)
        b2 = conv(x, cin, 192, 1)
        b2 = conv(b2, 192, 192, 1, kw=7, pad=3)
        b2 = conv(b2, 192, 192, 7, kw=1, pad=3)
        b2 = conv(b2, 192, 192, 3, stride=2)
        b3 = m.add(MAXPOOL, x, k=3, stride=2, pad=0)
        return cat([(b1, 320), (b2, 192), (b3, cin)])

    def block_e(x, cin):
        b1 = conv(x, cin, 320, 1)
        t = conv(x, cin, 384, 1)
        b2 = cat([(conv(t, 384, 384, 1, kw=3, pad=1), 384), (conv(t, 384, 384, 3, kw=1, pad=1), 384)])
        t = conv(conv(x, cin, 448, 1), 448, 384, 3, pad=1)
        b3 = cat([(conv(t, 384, 384, 1, kw=3, pad=1), 384), (conv(t, 384, 384, 3, kw=1, pad=1), 384)])
        b4 = conv(m.add(AVGPOOL, x, k=3, stride=1, pad=1), cin, 192, 1)
        return cat([(b1, 320), b2, b3, (b4, 192)])

    x = conv(MODEL_INPUT, 3, 32, 3, stride=2)
    x = conv(x, 32, 32, 3)
    x = conv(x, 32, 64, 3, pad=1)
    x = m.add(MAXPOOL, x, k=3, stride=2, pad=0)
    x = conv(x, 64, 80, 1)
    x = conv(x, 80, 192, 3)
    x = m.add(MAXPOOL, x, k=3, stride=2, pad=0)
    c = 192
    for pf in (32, 64, 64):
        x, c = block_a(x, c, pf)
    x, c = block_b(x, c)
    for c7 in (128, 160, 160, 192):
        x, c = block_c(x, c, c7)
    x, c = block_d(x, c)
    for _ in range(2):
        x, c = block_e(x, c)
    x = m.add(GAP, x)
    m.add(FC, x, cin=c, cout=classes)
    return m.shapes()


def _densenet(name: str, growth: int, blocks, init: int, dtype: str, classes: int, hw: int) -> Model:
    """DenseNet-BC (Huang et al. 2017): every dense layer normalises and rectifies the concatenation of all
    earlier features (a per-channel scale and shift: a 1x1 depthwise node here, it cannot be folded because
    every consumer has its own), squeezes it to 4*growth channels (1x1, its BatchNorm folded), adds `growth`
    new channels (3x3, no bias) and concatenates them; transitions halve channels (1x1, no bias) and size
    (2x2 average pooling)."""
    m = Model(name, dtype, 3, hw, hw)
    x = m.add(CONV, MODEL_INPUT, cin=3, cout=init, k=7, stride=2, pad=3, act=RELU)
    x = m.add(MAXPOOL, x, k=3, stride=2, pad=1)
    c = init
    for bi, n in enumerate(blocks):
        for _ in range(n):
            a = m.add(DWCONV, x, cin=c, cout=c, k=1, stride=1, pad=0, act=RELU, bn=False)
            a = m.add(CONV, a, cin=c, cout=4 * growth, k=1, stride=1, pad=0, act=RELU)
            a = m.add(CONV, a, cin=4 * growth, cout=growth, k=3, stride=1, pad=1, act=NONE, bias=False, bn=False)
            x = m.add(CONCAT, x, residual=a)
            c += growth
        if bi + 1 < len(blocks):
            a = m.add(DWCONV, x, cin=c, cout=c, k=1, stride=1, pad=0, act=RELU, bn=False)
            a = m.add(CONV, a, cin=c, cout=c // 2, k=1, stride=1, pad=0, act=NONE, bias=False, bn=False)
            x = m.add(AVGPOOL, a, k=2, stride=2, pad=0)
            c //= 2
    x = m.add(DWCONV, x, cin=c, cout=c, k=1, stride=1, pad=0, act=RELU, bn=False)
    x = m.add(GAP, x)
    m.add(FC, x, cin=c, cout=classes)
    return m.shapes()


def densenet121(dtype: str = "bf16", classes: int = 1000, hw: int = 224) -> Model:
    return _densenet("densenet121", 32, (6, 12, 24, 16), 64, dtype, classes, hw)


def densenet169(dtype: str = "bf16", classes: int = 1000, hw: int = 224) -> Model:
    return _densenet("densenet169", 32, (6, 12, 32, 32), 64, dtype, classes, hw)


def densenet201(dtype: str = "bf16", classes: int = 1000, hw: int = 224) -> Model:
    return _densenet("densenet201", 32, (6, 12, 48, 32), 64, dtype, classes, hw)


def densenet161(dtype: str = "bf16", classes: int = 1000, hw: int = 224) -> Model:
    return _densenet("densenet161", 48, (6, 12, 36, 24), 96, dtype, classes, hw)


def squeezenet1_0(dtype: str = "bf16", classes: int = 1000, hw: int = 224) -> Model:
    """SqueezeNet 1.0 (Iandola et al. 2016, Table 1): 7x7/2 stem with 96 channels, pooling after fire 4 and fire 8."""
    m = Model("squeezenet1_0", dtype, 3, hw, hw)
    x = m.add(CONV, MODEL_INPUT, cin=3, cout=96, k=7, stride=2, pad=0, act=RELU)
    x = m.add(MAXPOOL, x, k=3, stride=2, pad=0, ceil=True)
    cin = 96
    for idx, (sq, ex) in enumerate(((16, 64), (16, 64), (32, 128), (32, 128), (48, 192), (48, 192), (64, 256), (64, 256))):
        if idx in (3, 7):
            x = m.add(MAXPOOL, x, k=3, stride=2, pad=0, ceil=True)
        q = m.add(CONV, x, cin=cin, cout=sq, k=1, stride=1, pad=0, act=RELU)
        e1 = m.add(CONV, q, cin=sq, cout=ex, k=1, stride=1, pad=0, act=RELU)
        e3 = m.add(CONV, q, cin=sq, cout=ex, k=3, stride=1, pad=1, act=RELU)
        x = m.add(CONCAT, e1, residual=e3)
        cin = 2 * ex
    x = m.add(CONV, x, cin=512, cout=classes, k=1, stride=1, pad=0, act=RELU)
    m.add(GAP, x)
    return m.shapes()


def googlenet(dtype: str = "bf16", classes: int = 1000, hw: int = 224) -> Model:
    """GoogLeNet / Inception v1 (Szegedy et al. 2015) in its BatchNorm form without auxiliary heads: every
    inception module concatenates a 1x1 branch, a 1x1 -> 3x3 branch, a second 1x1 -> 3x3 branch (the widely
    used implementation's stand-in for the 5x5) and a 3x3/1 max pool -> 1x1 branch."""
    m = Model("googlenet", dtype, 3, hw, hw)

    def inception(x, cin, c1, c3r, c3, c5r, c5, cp):
        b1 = m.add(CONV, x, cin=cin, cout=c1, k=1, stride=1, pad=0, act=RELU)
        b2 = m.add(CONV, x, cin=cin, cout=c3r, k=1, stride=1, pad=0, act=RELU)
        b2 = m.add(CONV, b2, cin=c3r, cout=c3, k=3, stride=1, pad=1, act=RELU)
        b3 = m.add(CONV, x, cin=cin, cout=c5r, k=1, stride=1, pad=0, act=RELU)
        b3 = m.add(CONV, b3, cin=c5r, cout=c5, k=3, stride=1, pad=1, act=RELU)
        b4 = m.add(MAXPOOL, x, k=3, stride=1, pad=1, ceil=True)
        b4 = m.add(CONV, b4, cin=cin, cout=cp, k=1, stride=1, pad=0, act=RELU)
        y = m.add(CONCAT, b1, residual=b2)
        y = m.add(CONCAT, y, residual=b3)
        return m.add(CONCAT, y, residual=b4), c1 + c3 + c5 + cp

    x = m.add(CONV, MODEL_INPUT, cin=3, cout=64, k=7, stride=2, pad=3, act=RELU)
    x = m.add(MAXPOOL, x, k=3, stride=2, pad=0, ceil=True)
    x = m.add(CONV, x, cin=64, cout=64, k=1, stride=1, pad=0, act=RELU)
    x = m.add(CONV, x, cin=64, cout=192, k=3, stride=1, pad=1, act=RELU)
    x = m.add(MAXPOOL, x, k=3, stride=2, pad=0, ceil=True)
    c = 192
    for cfg in ((64, 96, 128, 16, 32, 32), (128, 128, 192, 32, 96, 64)):
        x, c = inception(x, c, *cfg)
    x = m.add(MAXPOOL, x, k=3, stride=2, pad=0, ceil=True)
    for cfg in ((192, 96, 208, 16, 48, 64), (160, 112, 224, 24, 64, 64), (128, 128, 256, 24, 64, 64),
                (112, 144, 288, 32, 64, 64), (256, 160, 320, 32, 128, 128)):
        x, c = inception(x, c, *cfg)
    x = m.add(MAXPOOL, x, k=2, stride=2, pad=0, ceil=True)
    for cfg in ((256, 160, 320, 32, 128, 128), (384, 192, 384, 48, 128, 128)):
        x, c = inception(x, c, *cfg)
    x = m.add(GAP, x)
    m.add(FC, x, cin=1024, cout=classes)
    return m.shapes()


FAMILIES = {"tiny": tiny_cnn, "resnet18": resnet18, "resnet50": resnet50,
            "mobilenetv2": mobilenetv2, "vgg16": vgg16,
            # further families of the paper's Table III that need no operator beyond the five above
            "alexnet": alexnet, "vgg11": vgg11, "vgg13": vgg13, "vgg19": vgg19,
            "resnet34": resnet34, "resnet101": resnet101, "resnet152": resnet152,
            "wide_resnet50_2": wide_resnet50_2, "wide_resnet101_2": wide_resnet101_2, "mnasnet1_0": mnasnet1_0,
            # ... and two that add channel concatenation and pooling sizes that round up
            "squeezenet1_0": squeezenet1_0, "squeezenet1_1": squeezenet1_1, "googlenet": googlenet,
            # ... and grouped convolution
            "resnext50_32x4d": resnext50_32x4d, "resnext101_32x8d": resnext101_32x8d,
            # ... and window average pooling with per-channel affine nodes
            # ... and squeeze-excite gates with hard-swish / hard-sigmoid activations
            "mobilenet_v3_large": mobilenet_v3_large, "mobilenet_v3_small": mobilenet_v3_small,
            "efficientnet_v2_s": efficientnet_v2_s, "efficientnet_v2_m": efficientnet_v2_m, "efficientnet_v2_l": efficientnet_v2_l,
            # ... and channel slices and shuffles
            "shufflenet_v2_x1_0": shufflenet_v2_x1_0, "shufflenet_v2_x0_5": shufflenet_v2_x0_5,
            # ... and rectangular kernels
            "inception_v3": inception_v3,
            "densenet121": densenet121, "densenet169": densenet169, "densenet201": densenet201, "densenet161": densenet161}
