"""Python face of the CPU oracle (ctypes over oracle/fi_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the benchmark's
cpu_baseline leg; never by the product package.  It knows nothing of the GPU
library: model descriptions arrive as `workloads.zoo.Model` data and are
translated here into the oracle's own `orc_layer` records.
"""
from __future__ import annotations

import ctypes as C
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

from . import build as _build

_HERE = os.path.dirname(os.path.abspath(__file__))
_OPS = {"conv": 0, "dwconv": 1, "maxpool": 2, "gap": 3, "fc": 4, "softmax": 5, "concat": 6, "avgpool": 7, "mul": 8, "slice": 9, "shuffle": 10}
_ACTS = {"none": 0, "relu": 1, "relu6": 2, "hardswish": 3, "hardsigmoid": 4, "silu": 5, "sigmoid": 6}
_DT = {"f32": 0, "bf16": 1}


class OrcLayer(C.Structure):
    _fields_ = [("op", C.c_int32), ("act", C.c_int32), ("input", C.c_int32), ("residual", C.c_int32),
                ("cin", C.c_int32), ("cout", C.c_int32), ("k", C.c_int32), ("stride", C.c_int32),
                ("pad", C.c_int32), ("ceil_mode", C.c_int32), ("w_off", C.c_int64), ("b_off", C.c_int64),
                ("groups", C.c_int32), ("c_first", C.c_int32),
                ("kw", C.c_int32), ("reserved", C.c_int32)]


_FP = C.POINTER(C.c_float)
_libs = {}


def lib(f64: bool = False):
    key = "f64" if f64 else "f32"
    if key not in _libs:
        _build.build(force=False)
        L = C.CDLL(os.path.join(_HERE, "liboracle_f64.so" if f64 else "liboracle.so"))
        L.orc_conv2d.argtypes = [_FP, C.c_int, C.c_int, C.c_int, C.c_int, _FP, _FP, C.c_int, C.c_int, C.c_int, C.c_int, _FP]
        L.orc_conv2d_grouped.argtypes = [_FP, C.c_int, C.c_int, C.c_int, C.c_int, _FP, _FP, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, _FP]
        L.orc_maxpool2d_ex.argtypes = [_FP, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, _FP]
        L.orc_avgpool2d.argtypes = [_FP, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, _FP]
        L.orc_channel_scale.argtypes = [_FP, _FP, C.c_int, C.c_int, C.c_int, C.c_int, _FP]
        L.orc_slice.argtypes = [_FP, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, _FP]
        L.orc_channel_shuffle.argtypes = [_FP, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, _FP]
        L.orc_conv2d_rect.argtypes = [_FP, C.c_int, C.c_int, C.c_int, C.c_int, _FP, _FP, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, _FP]
        L.orc_concat.argtypes = [_FP, C.c_int, _FP, C.c_int, C.c_int, C.c_int, C.c_int, _FP]
        L.orc_dwconv2d.argtypes = [_FP, C.c_int, C.c_int, C.c_int, C.c_int, _FP, _FP, C.c_int, C.c_int, C.c_int, _FP]
        L.orc_maxpool2d.argtypes = [_FP, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, _FP]
        L.orc_global_avgpool.argtypes = [_FP, C.c_int, C.c_int, C.c_int, C.c_int, _FP]
        L.orc_fc.argtypes = [_FP, C.c_int, C.c_int, _FP, _FP, C.c_int, _FP]
        L.orc_softmax.argtypes = [_FP, C.c_int, C.c_int, _FP]
        L.orc_top1.argtypes = [_FP, C.c_int, C.c_int, C.POINTER(C.c_int32)]
        L.orc_activate.argtypes = [_FP, C.c_int64, C.c_int]
        L.orc_add.argtypes = [_FP, _FP, C.c_int64]
        L.orc_round_bf16.argtypes = [_FP, C.c_int64]
        L.orc_bf16_round.argtypes = [C.c_float]
        L.orc_bf16_round.restype = C.c_float
        L.orc_run_model.argtypes = [C.POINTER(OrcLayer), C.c_int, C.c_int, C.c_void_p, C.c_int, _FP,
                                    C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, _FP, C.c_int64]
        L.orc_run_model.restype = C.c_int64
        L.orc_acc_bytes.restype = C.c_int
        _libs[key] = L
    return _libs[key]


def _f(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(_FP)


def _osz(n, k, s, p):
    return (n + 2 * p - k) // s + 1


def conv2d(x, w, b, stride=1, pad=0, f64=False):
    x, xp = _f(x); w, wp = _f(w)
    n, c, h, ww = x.shape
    o, ci, k, _ = w.shape
    assert ci == c
    bp = None
    if b is not None:
        b, bp = _f(b)
    y = np.empty((n, o, _osz(h, k, stride, pad), _osz(ww, k, stride, pad)), dtype=np.float32)
    lib(f64).orc_conv2d(xp, n, c, h, ww, wp, bp, o, k, stride, pad, y.ctypes.data_as(_FP))
    return y


def conv2d_rect(x, w, b, stride=1, pad_h=0, pad_w=0, f64=False):
    x, xp = _f(x); w, wp = _f(w)
    n, c, h, ww = x.shape
    o, ci, kh, kw = w.shape
    assert ci == c
    bp = None
    if b is not None:
        b, bp = _f(b)
    y = np.empty((n, o, _osz(h, kh, stride, pad_h), _osz(ww, kw, stride, pad_w)), dtype=np.float32)
    lib(f64).orc_conv2d_rect(xp, n, c, h, ww, wp, bp, o, kh, kw, stride, pad_h, pad_w, y.ctypes.data_as(_FP))
    return y


def conv2d_grouped(x, w, b, groups, stride=1, pad=0, f64=False):
    x, xp = _f(x); w, wp = _f(w)
    n, c, h, ww = x.shape
    o, ci, k, _ = w.shape
    assert ci * groups == c and o % groups == 0
    bp = None
    if b is not None:
        b, bp = _f(b)
    y = np.empty((n, o, _osz(h, k, stride, pad), _osz(ww, k, stride, pad)), dtype=np.float32)
    lib(f64).orc_conv2d_grouped(xp, n, c, h, ww, wp, bp, o, k, stride, pad, groups, y.ctypes.data_as(_FP))
    return y


def dwconv2d(x, w, b, stride=1, pad=0, f64=False):
    x, xp = _f(x); w, wp = _f(w)
    n, c, h, ww = x.shape
    k = w.shape[-1]
    bp = None
    if b is not None:
        b, bp = _f(b)
    y = np.empty((n, c, _osz(h, k, stride, pad), _osz(ww, k, stride, pad)), dtype=np.float32)
    lib(f64).orc_dwconv2d(xp, n, c, h, ww, wp, bp, k, stride, pad, y.ctypes.data_as(_FP))
    return y


def _osz_ceil(n, k, stride, pad):
    out = -((n + 2 * pad - k) // -stride) + 1
    return out - 1 if (out - 1) * stride >= n + pad else out


def maxpool2d(x, k, stride, pad=0, ceil=False):
    x, xp = _f(x)
    n, c, h, w = x.shape
    osz = _osz_ceil if ceil else _osz
    y = np.empty((n, c, osz(h, k, stride, pad), osz(w, k, stride, pad)), dtype=np.float32)
    lib().orc_maxpool2d_ex(xp, n, c, h, w, k, stride, pad, int(ceil), y.ctypes.data_as(_FP))
    return y


def avgpool2d(x, k, stride, pad=0, f64=False):
    x, xp = _f(x)
    n, c, h, w = x.shape
    y = np.empty((n, c, _osz(h, k, stride, pad), _osz(w, k, stride, pad)), dtype=np.float32)
    lib(f64).orc_avgpool2d(xp, n, c, h, w, k, stride, pad, y.ctypes.data_as(_FP))
    return y


def channel_scale(x, g):
    x, xp = _f(x)
    g, gp = _f(g)
    n, c, h, w = x.shape
    assert g.size == n * c
    y = np.empty_like(x)
    lib().orc_channel_scale(xp, gp, n, c, h, w, y.ctypes.data_as(_FP))
    return y


def channel_slice(x, first, count):
    x, xp = _f(x)
    n, c, h, w = x.shape
    y = np.empty((n, count, h, w), dtype=np.float32)
    lib().orc_slice(xp, n, c, h, w, first, count, y.ctypes.data_as(_FP))
    return y


def channel_shuffle(x, groups):
    x, xp = _f(x)
    n, c, h, w = x.shape
    y = np.empty_like(x)
    lib().orc_channel_shuffle(xp, n, c, h, w, groups, y.ctypes.data_as(_FP))
    return y


def concat(a, b):
    a, ap = _f(a)
    b, bp = _f(b)
    n, ca, h, w = a.shape
    assert b.shape[0] == n and b.shape[2:] == (h, w)
    y = np.empty((n, ca + b.shape[1], h, w), dtype=np.float32)
    lib().orc_concat(ap, ca, bp, b.shape[1], n, h, w, y.ctypes.data_as(_FP))
    return y


def global_avgpool(x, f64=False):
    x, xp = _f(x)
    n, c, h, w = x.shape
    y = np.empty((n, c), dtype=np.float32)
    lib(f64).orc_global_avgpool(xp, n, c, h, w, y.ctypes.data_as(_FP))
    return y


def fc(x, w, b, f64=False):
    x, xp = _f(x); w, wp = _f(w)
    n, i = x.shape
    o = w.shape[0]
    bp = None
    if b is not None:
        b, bp = _f(b)
    y = np.empty((n, o), dtype=np.float32)
    lib(f64).orc_fc(xp, n, i, wp, bp, o, y.ctypes.data_as(_FP))
    return y


def softmax(z, f64=False):
    z, zp = _f(z)
    n, k = z.shape
    p = np.empty((n, k), dtype=np.float32)
    lib(f64).orc_softmax(zp, n, k, p.ctypes.data_as(_FP))
    return p


def top1(z):
    z, zp = _f(z)
    n, k = z.shape
    idx = np.empty(n, dtype=np.int32)
    lib().orc_top1(zp, n, k, idx.ctypes.data_as(C.POINTER(C.c_int32)))
    return idx


def activate(y, act):
    y = np.array(y, dtype=np.float32, copy=True)
    lib().orc_activate(y.ctypes.data_as(_FP), y.size, _ACTS[act])
    return y


def round_bf16(y):
    y = np.array(y, dtype=np.float32, copy=True)
    lib().orc_round_bf16(y.ctypes.data_as(_FP), y.size)
    return y


def layer_table(model):
    arr = (OrcLayer * len(model.layers))()
    for i, L in enumerate(model.layers):
        arr[i] = OrcLayer(_OPS[L.op], _ACTS[L.act], L.input, L.residual, L.cin, L.cout, L.k, L.stride,
                          L.pad, int(getattr(L, "ceil", False)), L.w_off, L.b_off, int(getattr(L, "groups", 1)), int(getattr(L, "first", 0)),
                          int(getattr(L, "kw", 0)), 0)
    return arr


def out_elems(model, node=None):
    L = model.layers[model.output if node is None else node]
    return L.cout * L.out_h * L.out_w


def run_model(model, blob, x_nchw, round_storage=False, node=None, f64=False):
    """One model alone on a logical NCHW fp32 batch -> [N, elems of output node]."""
    x, xp = _f(x_nchw)
    n, c, h, w = x.shape
    node = model.output if node is None else node
    per = out_elems(model, node)
    out = np.empty((n, per), dtype=np.float32)
    tab = layer_table(model)
    blob = np.ascontiguousarray(blob)
    r = lib(f64).orc_run_model(tab, len(model.layers), model.output, blob.ctypes.data, _DT[model.dtype], xp,
                               n, c, h, w, 1 if round_storage else 0, node, out.ctypes.data_as(_FP), out.size)
    if r != out.size:
        raise RuntimeError(f"oracle failed: code {r}")
    return out


def run_models_parallel(units, threads=None):
    """units: list of (model, blob, x_nchw[1 image or more], round_storage).  Runs the
    single-threaded oracle on independent units concurrently (one unit per thread);
    returns outputs in order."""
    threads = threads or min(len(units), os.cpu_count() or 1)
    lib()
    with ThreadPoolExecutor(max_workers=max(1, threads)) as ex:
        return list(ex.map(lambda u: run_model(u[0], u[1], u[2], u[3]), units))
