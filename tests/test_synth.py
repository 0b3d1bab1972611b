"""The seeded input generator: deterministic, bf16-representable, outlier channels as specified."""
import numpy as np

from paper_2506_04648_amd import synth


def test_deterministic_and_bf16_representable():
    w = synth.TINY
    q1, k1, v1 = synth.qkv_raster(w)
    q2, k2, v2 = synth.qkv_raster(w)
    assert q1.shape == (2, 4, 16, 16, 128) and q1.dtype == np.float32
    assert np.array_equal(q1, q2) and np.array_equal(k1, k2) and np.array_equal(v1, v2)
    assert not np.array_equal(q1, k1)
    for a in (q1, k1, v1):
        assert np.all((a.view(np.uint32) & 0xFFFF) == 0)
    q3, _, _ = synth.qkv_raster(w, call_index=1)
    assert not np.array_equal(q1, q3)
    qh, _, _ = synth.qkv_raster(w, heads=[1])
    assert np.array_equal(qh[0], q1[1])                      # heads are independent streams


def test_outlier_channels():
    w = synth.TINY
    q, _, _ = synth.qkv_raster(w)
    std = q[0].reshape(-1, 128).std(axis=0)
    assert int((std > 4).sum()) == w.n_outlier and abs(np.median(std) - 1.0) < 0.1


def test_round_to_bf16_ties_to_even():
    x = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -9, -3.1415927], dtype=np.float32)
    r = synth.round_to_bf16(x)
    assert r[0] == 1.0 and r[1] == np.float32(1.0 + 2.0 ** -6) and r[2] == 1.0
    assert abs(r[3] + 3.140625) < 1e-7
