"""Brute-force token-level reference used only to pin the oracle on tiny inputs.

Everything here works on the RASTER (t,h,w) grid with plain Python loops: no tile ordering, no
padding, no vectorised rounding.  FP8 rounding is a nearest-value search with exact rational
arithmetic.  It deliberately shares nothing with oracle/ beyond the table of e4m3 values, which it
rebuilds itself from the format definition.
"""
import math
from fractions import Fraction

import numpy as np


def e4m3_values():
    vals = []
    for code in range(0x7F):
        e, m = code >> 3, code & 7
        vals.append(Fraction(m, 512) if e == 0 else Fraction(8 + m, 8) * Fraction(2) ** (e - 7))
    return vals


_VALS = e4m3_values()


def nearest_e4m3(q: Fraction) -> Fraction:
    """Nearest e4m3 value to the exact rational q: ties to the even code, saturating at 448."""
    a = min(abs(q), Fraction(448))
    best, bestd = 0, None
    for c, v in enumerate(_VALS):
        dd = abs(v - a)
        if bestd is None or dd < bestd or (dd == bestd and c % 2 == 0):
            best, bestd = c, dd
    return _VALS[best] if q >= 0 else -_VALS[best]


def tile_of(t, h, w, tile):
    return (t // tile[0], h // tile[1], w // tile[2])


def in_window(tu, tv, window):
    """Eq. 2 with tile centres c = index + 1/2 in tile units and the window in tiles:
    |c_u - c_v| <= w/2 on every axis."""
    return all(abs((tu[a] + 0.5) - (tv[a] + 0.5)) <= window[a] / 2.0 for a in range(3))


def quantize_raster(x, tile, per_channel=False):
    """x float64 [T,H,W,d] -> (dequantised values as float64 array, dict/array of scales)."""
    T, H, W, d = x.shape
    out = np.zeros_like(x)
    if per_channel:
        scales = np.zeros(d, dtype=np.float32)
        for c in range(d):
            amax = np.float32(np.abs(x[..., c]).max())
            s = np.float32(1.0) if amax == 0 else np.float32(amax) / np.float32(448.0)
            scales[c] = s
            for t in range(T):
                for h in range(H):
                    for w in range(W):
                        qv = nearest_e4m3(Fraction(float(x[t, h, w, c])) / Fraction(float(s)))
                        out[t, h, w, c] = float(qv * Fraction(float(s)))
        return out, scales
    scales = {}
    nT, nH, nW = -(-T // tile[0]), -(-H // tile[1]), -(-W // tile[2])
    for ut in range(nT):
        for uh in range(nH):
            for uw in range(nW):
                blk = x[ut * tile[0]:(ut + 1) * tile[0], uh * tile[1]:(uh + 1) * tile[1],
                        uw * tile[2]:(uw + 1) * tile[2]]
                amax = np.float32(np.abs(blk).max()) if blk.size else np.float32(0)
                s = np.float32(1.0) if amax == 0 else np.float32(amax) / np.float32(448.0)
                scales[(ut, uh, uw)] = s
    for t in range(T):
        for h in range(H):
            for w in range(W):
                s = Fraction(float(scales[tile_of(t, h, w, tile)]))
                for c in range(d):
                    out[t, h, w, c] = float(nearest_e4m3(Fraction(float(x[t, h, w, c])) / s) * s)
    return out, scales


def attention_raster(q, k, v, tile, window, fp8, v_per_channel=False, qtile=None):
    """One head, raster [T,H,W,d] float64 in and out.  qtile: quantisation sub-tile (it divides
    the tile, so the sub-tiles of all tiles together are simply the grid cut into qtile boxes);
    the window keeps counting in whole tiles."""
    T, H, W, d = q.shape
    if fp8:
        qt = tile if qtile is None else qtile
        qh, _ = quantize_raster(q, qt)
        kh, _ = quantize_raster(k, qt)
        vh, _ = quantize_raster(v, qt, per_channel=v_per_channel)
    else:
        qh, kh, vh = q, k, v
    toks = [(t, h, w) for t in range(T) for h in range(H) for w in range(W)]
    out = np.zeros_like(q)
    for (t, h, w) in toks:
        tu = tile_of(t, h, w, tile)
        keys = [kk for kk in toks if in_window(tu, tile_of(*kk, tile), window)]
        s2 = [float(np.dot(qh[t, h, w], kh[kk])) / math.sqrt(d) * math.log2(math.e) for kk in keys]
        m = math.ceil(max(s2))
        p = [2.0 ** (x - m) for x in s2]
        l = sum(p)
        acc = np.zeros(d)
        for pj, kk in zip(p, keys):
            if fp8:
                pj = float(nearest_e4m3(Fraction(448.0 * pj))) / 448.0
            acc += pj * vh[kk]
        out[t, h, w] = acc / l
    return out
