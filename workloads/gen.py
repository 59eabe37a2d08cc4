"""Seeded generators for weights, inputs and the request stream (data only).

Every tensor is drawn from a counter-based Philox stream keyed by
(seed, tensor id) and filled in its *logical* element order (OIHW weights,
NCHW inputs), so the values do not depend on any executor's storage layout.
For bf16 models the drawn values are rounded to bf16 once, here: the rounded
values *are* the model, and both executors consume identical numbers.

Canonical weight blob of a model (what both executors are handed):
for every conv / depthwise / FC node, in node order,
  weights  [cout][cin_per_group][k][k]  (FC: [cout][cin], cin in C,H,W order)
           stored in the model dtype (fp32, or bf16 as raw 16-bit patterns)
  bias     [cout] fp32
each tensor starting on a 64-byte boundary; `Layer.w_off` / `Layer.b_off` are
byte offsets into the blob.
"""
from __future__ import annotations

import numpy as np

from . import zoo

ALIGN = 64


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns, round-to-nearest-even (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


CHUNK = 1 << 20  # elements per Philox sub-stream
_POOL = None


def _pool():
    global _POOL
    if _POOL is None:
        from concurrent.futures import ThreadPoolExecutor
        import os
        _POOL = ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1))
    return _POOL


def _stream(seed: int, tensor_id: int, chunk: int = 0) -> np.random.Generator:
    # Philox-4x64: 128-bit key = (seed, tensor id); the 256-bit counter's third
    # word selects the chunk, so chunk j of a tensor is an independent stream
    # that any number of worker threads can fill in any order.
    return np.random.Generator(np.random.Philox(key=[int(seed), int(tensor_id)], counter=[0, 0, int(chunk), 0]))


def _normal_into(seed: int, tensor_id: int, n: int, std: float, dst: np.ndarray, as_bf16: bool) -> None:
    """Fill dst (float32[n] or uint16[n]) with std * N(0,1), element i of the
    tensor always coming from chunk i // CHUNK, position i % CHUNK."""
    def work(j):
        lo = j * CHUNK
        m = min(CHUNK, n - lo)
        v = _stream(seed, tensor_id, j).standard_normal(m, dtype=np.float32)
        v *= np.float32(std)
        dst[lo:lo + m] = bf16_bits(v) if as_bf16 else v
    nchunks = (n + CHUNK - 1) // CHUNK
    if nchunks <= 1:
        for j in range(nchunks):
            work(j)
    else:
        list(_pool().map(work, range(nchunks)))


def _align(n: int) -> int:
    return (n + ALIGN - 1) // ALIGN * ALIGN


def layout_blob(model: zoo.Model) -> int:
    """Assign w_off / b_off for every weighted node; return the blob size."""
    esz = 4 if model.dtype == "f32" else 2
    off = 0
    for L in model.layers:
        if L.op == zoo.CONV:
            nw = L.cout * (L.cin // L.groups) * L.k * (L.kw or L.k)
        elif L.op == zoo.DWCONV:
            nw = L.cout * L.k * L.k
        elif L.op == zoo.FC:
            nw = L.cout * L.cin
        else:
            continue
        L.w_off = off
        off = _align(off + nw * esz)
        L.b_off = off
        off = _align(off + L.cout * 4)
    return off


def make_blob(model: zoo.Model, seed: int, bias_std: float = 0.1, out: np.ndarray | None = None) -> np.ndarray:
    """He-normal weights (std = sqrt(2 / fan_in), fan_in = k*k*cin/groups, FC:
    cin), biases bias_std * N(0,1) in fp32 (0 => all-zero biases)."""
    size = layout_blob(model)
    blob = out if out is not None else np.zeros(size, dtype=np.uint8)
    assert blob.nbytes >= size
    for i, L in enumerate(model.layers):
        if L.op == zoo.CONV:
            kk = L.k * (L.kw or L.k)
            fan_in, nw = (L.cin // L.groups) * kk, L.cout * (L.cin // L.groups) * kk
        elif L.op == zoo.DWCONV:
            fan_in, nw = L.k * L.k, L.cout * L.k * L.k
        elif L.op == zoo.FC:
            fan_in, nw = L.cin, L.cout * L.cin
        else:
            continue
        std = float(np.sqrt(2.0 / fan_in))
        if model.dtype == "f32":
            _normal_into(seed, 2 * i, nw, std, blob[L.w_off:L.w_off + 4 * nw].view(np.float32), False)
        else:
            _normal_into(seed, 2 * i, nw, std, blob[L.w_off:L.w_off + 2 * nw].view(np.uint16), True)
        bview = blob[L.b_off:L.b_off + 4 * L.cout].view(np.float32)
        if bias_std > 0 and L.bias:
            _normal_into(seed, 2 * i + 1, L.cout, bias_std, bview, False)
        else:
            bview[:] = 0
    return blob


def make_input(seed: int, n: int, c: int, h: int, w: int, dist: str, dtype: str) -> np.ndarray:
    """Logical NCHW fp32 batch; values already rounded to the model dtype."""
    g = _stream(seed, 0xFFFF)
    if dist == "uniform":
        x = g.random((n, c, h, w), dtype=np.float32)
    elif dist == "normal":
        x = g.standard_normal((n, c, h, w), dtype=np.float32)
    else:
        raise ValueError(dist)
    if dtype == "bf16":
        x = bf16_to_f32(bf16_bits(x)).reshape(n, c, h, w)
    return x


def to_nhwc_storage(x_nchw: np.ndarray, dtype: str) -> np.ndarray:
    """The same values in the storage format device buffers use at the library
    boundary: NHWC, fp32 or raw bf16 bit patterns (exact, values are bf16)."""
    x = np.ascontiguousarray(np.transpose(x_nchw, (0, 2, 3, 1)))
    return x if dtype == "f32" else bf16_bits(x).reshape(x.shape)


def request_stream(seed: int, n_requests: int, pool_size: int, subset: int,
                   rate_hz: float, n_input_batches: int):
    """Poisson arrivals: exponential inter-arrival times at `rate_hz`; every
    request picks `subset` distinct pool members uniformly and one of
    `n_input_batches` pre-generated input batches."""
    g = _stream(seed, 0xABCD)
    t = np.cumsum(g.exponential(1.0 / rate_hz, n_requests))
    reqs = []
    for i in range(n_requests):
        members = sorted(int(v) for v in g.choice(pool_size, size=subset, replace=False))
        reqs.append((float(t[i]), members, int(g.integers(n_input_batches))))
    return reqs
