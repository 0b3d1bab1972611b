"""Pins for the oracle's e4m3 codec: format definition, round trip, ties, scaled encode."""
import os

import numpy as np
import pytest

from oracle import e4m3

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "e4m3_known_codes.txt")


def _golden_rows():
    rows = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            v, c = line.split()
            rows.append((float(v), int(c, 16)))
    return rows


def test_known_codes_from_format_definition():
    for value, code in _golden_rows():
        got = int(e4m3.encode(np.array([value]))[0])
        assert got == code, (value, hex(got), hex(code))
        if abs(value) <= 448 and e4m3.decode(np.array([code]))[0] == value:
            assert e4m3.round_to_e4m3(np.array([value]))[0] == value


def test_decode_table_is_the_format():
    vals = e4m3.decode(np.arange(256, dtype=np.uint8))
    assert np.isnan(vals[0x7F]) and np.isnan(vals[0xFF])
    finite = np.delete(vals, [0x7F, 0xFF])
    assert np.all(np.isfinite(finite)) and finite.max() == 448.0 and finite.min() == -448.0
    pos = vals[:0x7F]
    assert np.all(np.diff(pos) > 0)                       # codes are ordered like their values
    # every value is a multiple of 2^-9 with at most 4 significant bits
    for v in pos[1:]:
        m, _ = np.frexp(v)
        assert (m * 16) == int(m * 16) and (v * 512) == int(v * 512)
    assert pos.size == 127 and pos[1] == 2.0 ** -9 and pos[8] == 2.0 ** -6
    assert np.array_equal(vals[0x80:0xFF], -vals[0x00:0x7F])


def test_round_trip_all_finite_codes():
    codes = np.array([c for c in range(256) if c not in (0x7F, 0xFF)], dtype=np.uint8)
    vals = e4m3.decode(codes)
    back = e4m3.encode(vals)
    # +0 and -0 keep their sign bit; everything else must reproduce its code
    assert np.array_equal(back, codes)
    assert np.array_equal(e4m3.round_to_e4m3(vals), vals)


def _nearest_by_search(y):
    """Brute force: nearest table value, ties to the even code, saturating."""
    table = e4m3.decode(np.arange(0x7F, dtype=np.uint8))
    a = min(abs(y), 448.0)
    best, bestd = 0, None
    for c, v in enumerate(table):
        dd = abs(v - a)
        if bestd is None or dd < bestd or (dd == bestd and c % 2 == 0):
            best, bestd = c, dd
    return table[best] * (1.0 if y >= 0 else -1.0), best | (0x80 if np.signbit(y) else 0)


def test_both_encoders_agree_with_brute_force_search():
    rng = np.random.default_rng(7)
    table = e4m3.decode(np.arange(0x7F, dtype=np.uint8))
    mids = 0.5 * (table[:-1] + table[1:])
    ys = np.concatenate([mids, np.nextafter(mids, 0), np.nextafter(mids, 1e9), table,
                         rng.uniform(-460, 460, 2000), rng.normal(0, 0.01, 2000),
                         2.0 ** rng.uniform(-14, 9, 2000)])
    ys = np.concatenate([ys, -ys])
    vals = e4m3.round_to_e4m3(ys)
    codes = e4m3.encode(ys)
    for y, v, c in zip(ys, vals, codes):
        bv, bc = _nearest_by_search(float(y))
        assert v == bv, (y, v, bv)
        assert int(c) == bc or (bv == 0 and (int(c) & 0x7F) == 0), (y, hex(int(c)), hex(bc))
    assert np.array_equal(e4m3.decode(codes), vals)
    assert not np.any((codes & 0x7F) == 0x7F)              # NaN is never produced


def test_scaled_encode_exact_quotient_decides_ties():
    # s chosen so that x/s sits an ulp of float64 away from a midpoint: the exact comparison
    # against mid*s must still see which side it is on.
    s = float(np.float32(0.0123456789))
    for mid, lo_code in ((17.0, 0x58), (19.0, 0x59), (2.0 ** -10, 0x00), (416.0 + 16.0, 0x7D)):
        x = mid * s                                          # exact in float64 (5 x 24 bits)
        tie_code = int(e4m3.encode_scaled(np.array([x]), s)[0])
        assert tie_code in (lo_code, lo_code + 1) and tie_code % 2 == 0
        assert int(e4m3.encode_scaled(np.array([np.nextafter(x, 0)]), s)[0]) == lo_code
        assert int(e4m3.encode_scaled(np.array([np.nextafter(x, 1e9)]), s)[0]) == lo_code + 1
    # scale invariance: encode_scaled(x, s) == encode(x / s) whenever x/s is exact (s a power of 2)
    rng = np.random.default_rng(3)
    x = rng.normal(0, 3, 4096)
    for k in (-5, 0, 4):
        assert np.array_equal(e4m3.encode_scaled(x, 2.0 ** k), e4m3.encode(x / 2.0 ** k))


def test_relative_error_bound():
    # in the normal range the rounding error is at most half a spacing: 2^-4 relative
    y = 2.0 ** np.random.default_rng(5).uniform(-6, np.log2(448), 20000)
    r = e4m3.round_to_e4m3(y)
    assert np.max(np.abs(r - y) / y) <= 2.0 ** -4
    ysub = np.random.default_rng(6).uniform(0, 2.0 ** -6, 5000)
    assert np.max(np.abs(e4m3.round_to_e4m3(ysub) - ysub)) <= 2.0 ** -10
