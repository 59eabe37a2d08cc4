"""The seeded generators: determinism, distribution, layout independence."""
import hashlib

import numpy as np

from workloads import gen, zoo


def test_blob_deterministic_and_distinct_per_seed():
    m = zoo.resnet18(hw=64)
    a, b, c = gen.make_blob(m, 1000), gen.make_blob(m, 1000), gen.make_blob(m, 1001)
    assert hashlib.sha1(a.tobytes()).hexdigest() == hashlib.sha1(b.tobytes()).hexdigest()
    assert not np.array_equal(a, c)


def test_he_normal_statistics():
    m = zoo.vgg16(hw=32)
    blob = gen.make_blob(m, 3)
    L = m.layers[3]  # conv 64 -> 128
    nw = L.cout * L.cin * 9
    w = gen.bf16_to_f32(blob[L.w_off:L.w_off + 2 * nw].view(np.uint16))
    std = np.sqrt(2.0 / (9 * L.cin))
    assert abs(w.mean()) < 4 * std / np.sqrt(nw)
    assert abs(w.std() / std - 1) < 0.01
    b = blob[L.b_off:L.b_off + 4 * L.cout].view(np.float32)
    assert abs(b.std() - 0.1) < 0.03
    t = zoo.tiny_cnn()
    tb = gen.make_blob(t, 1000, bias_std=0.0)
    for L in t.layers:
        if L.op in ("conv", "fc"):
            assert not tb[L.b_off:L.b_off + 4 * L.cout].any()


def test_bf16_bits_roundtrip_and_input():
    x = gen.make_input(7, 2, 3, 16, 16, "normal", "bf16")
    assert np.array_equal(gen.bf16_to_f32(gen.bf16_bits(x)).reshape(x.shape), x)  # already bf16 values
    s = gen.to_nhwc_storage(x, "bf16")
    assert s.shape == (2, 16, 16, 3) and s.dtype == np.uint16
    assert np.array_equal(gen.bf16_to_f32(s).reshape(2, 16, 16, 3).transpose(0, 3, 1, 2), x)
    u = gen.make_input(7, 1, 3, 32, 32, "uniform", "f32")
    assert 0 <= u.min() and u.max() < 1 and abs(u.mean() - 0.5) < 0.02


def test_request_stream():
    r = gen.request_stream(2024, 1000, 16, 4, 50.0, 2)
    assert r == gen.request_stream(2024, 1000, 16, 4, 50.0, 2)
    ts = np.array([t for t, _, _ in r])
    assert np.all(np.diff(ts) > 0) and abs(np.diff(ts).mean() - 0.02) < 0.003
    assert all(len(set(mm)) == 4 and max(mm) < 16 for _, mm, _ in r)
    counts = np.bincount([i for _, mm, _ in r for i in mm], minlength=16)
    assert counts.min() > 180 and counts.max() < 320
