"""CPU oracle for FP8 3D sliding-tile attention -- TEST INFRASTRUCTURE ONLY.

A plain, slow float64 NumPy statement of what the hot path computes, written from the paper
(Sec. 3.1 Eq. 1-3, Sec. 3.2 Eq. 4-5, Sec. 3.3 Eq. 6, Algorithm 1).  Only tests, the smoke check
and the benchmark's cpu_baseline leg may import it.  It shares no code, table or helper with the
HIP path and never imports the product package.

Steps, in the paper's order (Algorithm 1):
  1. step-aware selection of (precision, window)                      -> schedule_select
  2. partition the (T,H,W) token grid into 3D tiles, made contiguous  -> tile_order / tile_unorder
  3. per-tile scale s = amax / 448 and FP8 encode of x / s            -> tile_scales / quantize_tiles
     (per-channel scales for V, the paper's own variant)              -> channel_scales / quantize_channels
  4. tile neighbourhood W(u) (Eq. 2) and masked softmax (Eq. 3)       -> tile_mask / attention
  5. P quantised with the fixed scale 1/448, PV, dequantise           -> attention

Readings taken where the paper is silent or garbled are listed in the design notes; the ones that
shape this file: scale = amax/448 applied as x/s (Eq. 4 decides the direction Eq. 1 leaves open);
window sizes are in tiles and a key tile is kept iff |u_a - v_a| <= floor(w_a/2) on every axis
(Eq. 2 with tile-index centres; truncated at the grid boundary); zero padding up to tile multiples,
padded keys excluded, padded query rows output 0; P is the un-normalised 2^(S' - m_i) with the row
reference m_i snapped up to an integer so that FP8 rounding of P does not depend on block order;
the softmax denominator is the sum of the un-quantised P.

Parity unpinned: the snapped reference and the un-quantised denominator are definitions of this
build, not derivable from the paper, and the paper prints no numeric example to compare with.
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np

from . import e4m3

LOG2E = math.log2(math.e)

PREC_BF16 = 0     # no quantisation: exact masked softmax attention on the given inputs
PREC_FP8 = 1      # Q, K, V and P in e4m3 (Sec. 3.2)
VSCALE_TILE = 0   # one V scale per 3D tile (the graded path)
VSCALE_CHANNEL = 1  # one V scale per channel over all tokens (the paper's Sec. 3.2 variant)


@dataclasses.dataclass(frozen=True)
class Geometry:
    """Token grid (T,H,W), tile (Tt,Th,Tw) and everything derived from them (Sec. 3.1).

    (Qt,Qh,Qw), if given, is the quantisation granularity g (Sec. 3.3 names g(t) and W(t) as
    separate hyper-parameters): each tile is cut into sub-tiles of that shape, which must divide
    the tile, and every sub-tile has its own scale, while the window of Eq. 2 keeps counting in
    whole tiles.  The default (0,0,0) is the unified granularity: one scale per tile."""
    T: int
    H: int
    W: int
    Tt: int
    Th: int
    Tw: int
    Qt: int = 0
    Qh: int = 0
    Qw: int = 0

    def __post_init__(self):
        qt, qh, qw = self.qtile
        assert self.Tt % qt == 0 and self.Th % qh == 0 and self.Tw % qw == 0, "sub-tile must divide the tile"

    @property
    def qtile(self):
        if self.Qt == 0 and self.Qh == 0 and self.Qw == 0:
            return (self.Tt, self.Th, self.Tw)
        return (self.Qt, self.Qh, self.Qw)

    @property
    def NS(self):
        """Quantisation groups (sub-tiles) per tile."""
        qt, qh, qw = self.qtile
        return (self.Tt // qt) * (self.Th // qh) * (self.Tw // qw)

    @property
    def n_groups(self):
        return self.M * self.NS

    @property
    def n_tiles_axis(self):
        return (-(-self.T // self.Tt), -(-self.H // self.Th), -(-self.W // self.Tw))

    @property
    def padded(self):
        nT, nH, nW = self.n_tiles_axis
        return (nT * self.Tt, nH * self.Th, nW * self.Tw)

    @property
    def M(self):
        nT, nH, nW = self.n_tiles_axis
        return nT * nH * nW

    @property
    def TS(self):
        return self.Tt * self.Th * self.Tw

    @property
    def L_real(self):
        return self.T * self.H * self.W

    @property
    def L_padded(self):
        return self.M * self.TS


# ----------------------------------------------------------------------------------------------
# Step 2: tile order (Sec. 3.2 step (1): tokens of one 3D tile become contiguous)
# ----------------------------------------------------------------------------------------------
def token_positions(g: Geometry) -> np.ndarray:
    """For every real token (t,h,w) in raster order, its position p = u*TS + r in the tile-ordered
    padded sequence: tile u = (ut*nH + uh)*nW + uw, in-tile rank r = ((t%Tt)*Th + h%Th)*Tw + w%Tw."""
    nT, nH, nW = g.n_tiles_axis
    t, h, w = np.meshgrid(np.arange(g.T), np.arange(g.H), np.arange(g.W), indexing="ij")
    u = ((t // g.Tt) * nH + (h // g.Th)) * nW + (w // g.Tw)
    r = ((t % g.Tt) * g.Th + (h % g.Th)) * g.Tw + (w % g.Tw)
    return (u * g.TS + r).reshape(-1)


def tile_order(x: np.ndarray, g: Geometry) -> np.ndarray:
    """[..., T, H, W, d] raster -> [..., M*TS, d] tile-ordered, zero in the padded slots."""
    lead = x.shape[:-4]
    d = x.shape[-1]
    assert x.shape[-4:-1] == (g.T, g.H, g.W)
    out = np.zeros(lead + (g.L_padded, d), dtype=x.dtype)
    out[..., token_positions(g), :] = x.reshape(lead + (g.L_real, d))
    return out


def tile_unorder(y: np.ndarray, g: Geometry) -> np.ndarray:
    """Inverse of tile_order on the real tokens: [..., M*TS, d] -> [..., T, H, W, d]."""
    lead = y.shape[:-2]
    return y[..., token_positions(g), :].reshape(lead + (g.T, g.H, g.W, y.shape[-1]))


def group_of_slot(g: Geometry) -> np.ndarray:
    """int [M*TS]: the quantisation group of every tile-ordered slot.  Slot (u, r) with in-tile
    coordinates (rt,rh,rw) belongs to sub-tile s = ((rt//Qt)*(Th//Qh) + rh//Qh)*(Tw//Qw) + rw//Qw
    of tile u, group u*NS + s.  With the unified granularity this is just the tile index."""
    qt, qh, qw = g.qtile
    r = np.arange(g.TS)
    rw, rh, rt = r % g.Tw, (r // g.Tw) % g.Th, r // (g.Tw * g.Th)
    s = ((rt // qt) * (g.Th // qh) + rh // qh) * (g.Tw // qw) + rw // qw
    return (np.arange(g.M)[:, None] * g.NS + s[None, :]).reshape(-1)


def valid_tokens(g: Geometry) -> np.ndarray:
    """bool [M*TS]: True where the tile-ordered slot holds a real token (t<T, h<H, w<W)."""
    v = np.zeros(g.L_padded, dtype=bool)
    v[token_positions(g)] = True
    return v


# ----------------------------------------------------------------------------------------------
# Step 4a: tile neighbourhood (Eq. 2)
# ----------------------------------------------------------------------------------------------
def tile_coords(g: Geometry) -> np.ndarray:
    nT, nH, nW = g.n_tiles_axis
    ut, uh, uw = np.meshgrid(np.arange(nT), np.arange(nH), np.arange(nW), indexing="ij")
    return np.stack([ut.reshape(-1), uh.reshape(-1), uw.reshape(-1)], axis=1)


EDGE_TRUNCATE = 0   # Eq. 2 as a pure distance test: edge tiles keep fewer key tiles
EDGE_SHIFT = 1      # the window centre is clamped into the grid: constant number of key tiles


def tile_mask(g: Geometry, window, edge=None) -> np.ndarray:
    """bool [M, M]: keep[u, v] iff the Chebyshev-type box test of Eq. 2 holds on every axis,
    with window sizes in tiles: |c_a - v_a| <= r_a = floor(w_a / 2).  The centre c is the query
    tile itself (truncating edges, the literal Eq. 2), or with edge == EDGE_SHIFT the query tile
    clamped to [r_a, n_a - 1 - r_a] so that the box never leaves the grid (an axis not longer than
    the window is kept whole).  `window` may carry the edge rule as a fourth entry."""
    if edge is None:
        edge = window[3] if len(window) > 3 else EDGE_TRUNCATE
    c = tile_coords(g)
    keep = np.ones((g.M, g.M), dtype=bool)
    for a, n in enumerate(g.n_tiles_axis):
        r = int(window[a]) // 2
        u, v = c[:, a][:, None], c[:, a][None, :]
        if edge == EDGE_SHIFT:
            if n <= 2 * r + 1:
                continue                                   # the window covers the whole axis
            centre = np.clip(u, r, n - 1 - r)
        else:
            centre = u
        keep &= np.abs(centre - v) <= r
    return keep


# ----------------------------------------------------------------------------------------------
# Step 3: scales and FP8 encode (Eq. 1, 4, 5)
# ----------------------------------------------------------------------------------------------
def _scale_from_amax(amax: np.ndarray) -> np.ndarray:
    """s = amax / 448 rounded once to float32 (float64 division then one rounding equals a
    correctly rounded float32 division); an all-zero group takes s = 1."""
    s = (np.asarray(amax, dtype=np.float64) / e4m3.FP8_MAX).astype(np.float32)
    return np.where(np.asarray(amax) == 0, np.float32(1.0), s).astype(np.float32)


def tile_scales(x_tiled: np.ndarray, g: Geometry) -> np.ndarray:
    """[..., M*TS, d] -> float32 [..., M*NS]: Eq. 4, max over all entries of each quantisation
    group (the whole tile, TS*d entries, unless the geometry names a finer sub-tile)."""
    lead = x_tiled.shape[:-2]
    d = x_tiled.shape[-1]
    if g.NS == 1:
        amax = np.abs(x_tiled.reshape(lead + (g.M, g.TS * d))).max(axis=-1)
        return _scale_from_amax(amax)
    grp = group_of_slot(g)
    row_amax = np.abs(x_tiled).max(axis=-1).reshape((-1, g.L_padded))
    amax = np.zeros((row_amax.shape[0], g.n_groups), dtype=row_amax.dtype)
    for b in range(row_amax.shape[0]):
        np.maximum.at(amax[b], grp, row_amax[b])
    return _scale_from_amax(amax.reshape(lead + (g.n_groups,)))


def channel_scales(x_tiled: np.ndarray) -> np.ndarray:
    """[..., L, d] -> float32 [..., d]: max over all tokens of each channel (Sec. 3.2, V)."""
    return _scale_from_amax(np.abs(x_tiled).max(axis=-2))


def quantize_tiles(x_tiled: np.ndarray, g: Geometry):
    """Per-group scales and e4m3 codes.  Returns (codes uint8 [..., M*TS, d], scales f32 [..., M*NS])."""
    scales = tile_scales(x_tiled, g)
    lead = x_tiled.shape[:-2]
    d = x_tiled.shape[-1]
    if g.NS == 1:
        xt = x_tiled.reshape((-1, g.M, g.TS * d))
        sc = scales.reshape((-1, g.M))
        codes = np.empty(xt.shape, dtype=np.uint8)
        for b in range(xt.shape[0]):
            for u in range(g.M):
                codes[b, u] = e4m3.encode_scaled(xt[b, u], sc[b, u])
        return codes.reshape(lead + (g.L_padded, d)), scales
    grp = group_of_slot(g)
    members = [np.flatnonzero(grp == i) for i in range(g.n_groups)]
    xt = x_tiled.reshape((-1, g.L_padded, d))
    sc = scales.reshape((-1, g.n_groups))
    codes = np.empty(xt.shape, dtype=np.uint8)
    for b in range(xt.shape[0]):
        for i, rows in enumerate(members):
            codes[b, rows] = e4m3.encode_scaled(xt[b, rows], sc[b, i])
    return codes.reshape(lead + (g.L_padded, d)), scales


def quantize_channels(x_tiled: np.ndarray):
    """Per-channel scales and codes (V in the paper's variant)."""
    scales = channel_scales(x_tiled)
    lead = x_tiled.shape[:-2]
    L, d = x_tiled.shape[-2:]
    xt = x_tiled.reshape((-1, L, d))
    sc = scales.reshape((-1, d))
    codes = np.empty(xt.shape, dtype=np.uint8)
    for b in range(xt.shape[0]):
        for c in range(d):
            codes[b, :, c] = e4m3.encode_scaled(xt[b, :, c], sc[b, c])
    return codes.reshape(lead + (L, d)), scales


# ----------------------------------------------------------------------------------------------
# Step 1: denoising-step-aware schedule (Eq. 6)
# ----------------------------------------------------------------------------------------------
def schedule_select(step: int, num_steps: int, alpha1: float, alpha2: float) -> int:
    """Index of the regime for 1-based step t of D: 0 if t <= a1*D, 1 if a1*D < t <= a2*D, else 2.
    The thresholds are evaluated in float32 like the C structure that carries them."""
    assert 1 <= step <= num_steps and 0.0 < alpha1 < alpha2 < 1.0
    t1 = float(np.float32(alpha1) * np.float32(num_steps))
    t2 = float(np.float32(alpha2) * np.float32(num_steps))
    if step <= t1:
        return 0
    if step <= t2:
        return 1
    return 2


# ----------------------------------------------------------------------------------------------
# Steps 4b-5: masked softmax attention with FP8 operands
# ----------------------------------------------------------------------------------------------
def attention(q_tiled, k_tiled, v_tiled, g: Geometry, window, prec=PREC_FP8, vscale=VSCALE_TILE,
              q_tiles=None, return_parts=False):
    """Attention output for ONE head.

    q_tiled, k_tiled, v_tiled: float64 (or float32) [M*TS, d], tile-ordered, zero padded.
    Returns O float64 [len(q_tiles)*TS, d] for the requested query tiles (default all), rows of
    padded query slots being 0.  With return_parts=True also returns, per requested query tile, the
    intermediate quantities (key columns, dequantised scores S', row reference m, un-normalised P,
    denominator l, quantised P, dequantised V rows, raw code dot products, the sums of their
    absolute products and the per-pair score scale) so that a comparator can inspect individual
    rounding decisions.
    """
    M, TS = g.M, g.TS
    d = q_tiled.shape[-1]
    q_tiles = list(range(M)) if q_tiles is None else list(q_tiles)
    keep = tile_mask(g, window)
    valid = valid_tokens(g)
    grp = group_of_slot(g)                                   # quantisation group of every slot
    c_scale = LOG2E / math.sqrt(d)

    if prec == PREC_FP8:
        qc, sq = quantize_tiles(np.asarray(q_tiled, dtype=np.float64), g)
        kc, sk = quantize_tiles(np.asarray(k_tiled, dtype=np.float64), g)
        qh, kh = e4m3.decode(qc), e4m3.decode(kc)           # unscaled code values
        if vscale == VSCALE_TILE:
            vc, sv = quantize_tiles(np.asarray(v_tiled, dtype=np.float64), g)
            vh = e4m3.decode(vc) * sv.astype(np.float64)[grp][:, None]
        else:
            vc, sv = quantize_channels(np.asarray(v_tiled, dtype=np.float64))
            vh = e4m3.decode(vc) * sv.astype(np.float64)[None, :]
        sq = sq.astype(np.float64)
        sk = sk.astype(np.float64)
    else:
        qh = np.asarray(q_tiled, dtype=np.float64)
        kh = np.asarray(k_tiled, dtype=np.float64)
        vh = np.asarray(v_tiled, dtype=np.float64)
        sq = np.ones(g.n_groups)
        sk = np.ones(g.n_groups)

    out = np.zeros((len(q_tiles) * TS, d), dtype=np.float64)
    parts = []
    for n, u in enumerate(q_tiles):
        vs = np.flatnonzero(keep[u])
        cols = (vs[:, None] * TS + np.arange(TS)[None, :]).reshape(-1)
        cols = cols[valid[cols]]                              # padded keys never take part
        Qu = qh[u * TS:(u + 1) * TS]
        Kw = kh[cols]
        # S' = (q.k) * s^Q * s^K * log2(e)/sqrt(d): scores dequantised per pair of quantisation
        # groups (per tile pair under the unified granularity), base 2
        raw = Qu @ Kw.T
        pair_scale = sq[grp[u * TS:(u + 1) * TS]][:, None] * sk[grp[cols]][None, :] * c_scale
        S = raw * pair_scale
        m = np.ceil(S.max(axis=1))                            # integer row reference
        p = np.exp2(S - m[:, None])                           # un-normalised P in (0, 1]
        l = p.sum(axis=1)                                     # denominator: un-quantised P
        if prec == PREC_FP8:
            ph = e4m3.round_to_e4m3(e4m3.FP8_MAX * p) / e4m3.FP8_MAX   # fixed scale 1/448 (Sec. 3.2)
        else:
            ph = p
        o = (ph @ vh[cols]) / l[:, None]
        rows_valid = valid[u * TS:(u + 1) * TS]
        o[~rows_valid] = 0.0
        out[n * TS:(n + 1) * TS] = o
        if return_parts:
            # sum_c |q_c k_c|: the yardstick against which a hardware accumulation error is measured
            absraw = np.abs(Qu) @ np.abs(Kw).T
            parts.append(dict(u=u, key_tiles=vs, cols=cols, raw=raw, absraw=absraw, pair_scale=pair_scale,
                              S=S, m=m, p=p, l=l, ph=ph, v=vh[cols], rows_valid=rows_valid))
    if return_parts:
        return out, parts
    return out
