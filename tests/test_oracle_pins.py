"""Pins for the attention oracle: closed forms, invariants, special cases, brute force."""
import math
import os

import numpy as np
import pytest
import scipy.special

from oracle import e4m3
from oracle import fps_oracle as fo
from tests import brute

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def bf16(x):
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    u = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return u.view(np.float32).astype(np.float64)


def rand_qkv(seed, grid, d, outlier=True):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((3,) + tuple(grid) + (d,))
    if outlier:
        x[0, ..., 1] *= 8
        x[1, ..., 2] *= 8
        x[2, ..., 0] *= 8
    x = bf16(x)
    return x[0], x[1], x[2]


SMALL = fo.Geometry(3, 5, 6, 2, 2, 4)        # pads to 4x6x8: 12 tiles of 16 tokens, ragged on all axes


# ---- tile order ---------------------------------------------------------------------------
def test_tile_order_is_a_permutation_with_zero_padding():
    g = SMALL
    x = np.arange(g.L_real * 2, dtype=np.float64).reshape(g.T, g.H, g.W, 2) + 1
    y = fo.tile_order(x, g)
    assert y.shape == (g.L_padded, 2) and g.L_padded == 4 * 6 * 8 and g.M == 12 and g.TS == 16
    assert np.array_equal(fo.tile_unorder(y, g), x)
    valid = fo.valid_tokens(g)
    assert valid.sum() == g.L_real and np.all(y[~valid] == 0) and np.all(y[valid] != 0)
    # explicit loop over raster coordinates
    nT, nH, nW = g.n_tiles_axis
    for t in range(g.T):
        for h in range(g.H):
            for w in range(g.W):
                u = ((t // g.Tt) * nH + h // g.Th) * nW + w // g.Tw
                r = ((t % g.Tt) * g.Th + h % g.Th) * g.Tw + w % g.Tw
                assert np.array_equal(y[u * g.TS + r], x[t, h, w])
    # tokens of one tile are contiguous: each tile's slots map back into one 3D box
    pos = fo.token_positions(g).reshape(g.T, g.H, g.W)
    assert set((pos[0:2, 0:2, 0:4] // g.TS).reshape(-1)) == {0}


# ---- tile mask (Eq. 2) --------------------------------------------------------------------
def _golden_pairs():
    rows = []
    with open(os.path.join(GOLDEN, "kept_tile_pairs.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                rows.append([int(x) for x in line.split()])
    return rows


@pytest.mark.parametrize("row", _golden_pairs())
def test_kept_pair_counts_closed_form(row):
    T, H, W, Tt, Th, Tw, wt, wh, ww, pairs = row
    g = fo.Geometry(T, H, W, Tt, Th, Tw)
    keep = fo.tile_mask(g, (wt, wh, ww))
    assert int(keep.sum()) == pairs
    closed = 1
    for n, w in zip(g.n_tiles_axis, (wt, wh, ww)):
        r = min(w // 2, n - 1)
        closed *= n * (2 * r + 1) - r * (r + 1)
    assert closed == pairs
    assert np.array_equal(keep, keep.T) and np.all(np.diag(keep))


@pytest.mark.parametrize("window", [(1, 1, 1), (1, 3, 3), (3, 3, 1), (2, 2, 2), (5, 6, 10), (6, 6, 1)])
def test_tile_mask_against_real_valued_centres(window):
    g = fo.Geometry(7, 9, 10, 1, 2, 3)
    keep = fo.tile_mask(g, window)
    nT, nH, nW = g.n_tiles_axis
    tiles = [(a, b, c) for a in range(nT) for b in range(nH) for c in range(nW)]
    for iu, tu in enumerate(tiles):
        for iv, tv in enumerate(tiles):
            assert keep[iu, iv] == brute.in_window(tu, tv, window)


@pytest.mark.parametrize("window", [(3, 3, 3), (5, 3, 1), (2, 7, 4), (9, 9, 99)])
def test_shifted_window_keeps_a_constant_number_of_tiles(window):
    g = fo.Geometry(7, 9, 10, 1, 2, 3)                       # 7 x 5 x 4 tiles
    keep = fo.tile_mask(g, window, edge=fo.EDGE_SHIFT)
    per_axis = [min(2 * (w // 2) + 1, n) for w, n in zip(window, g.n_tiles_axis)]
    assert np.all(keep.sum(axis=1) == per_axis[0] * per_axis[1] * per_axis[2])
    assert np.all(np.diag(keep))                             # a tile always sees itself
    trunc = fo.tile_mask(g, window)
    assert np.all(keep | ~trunc)                             # the truncated window is a subset
    # explicit definition per axis: a contiguous run of fixed length that contains u and fits the grid
    nT, nH, nW = g.n_tiles_axis
    tiles = [(a, b, c) for a in range(nT) for b in range(nH) for c in range(nW)]
    for iu, tu in enumerate(tiles):
        for iv, tv in enumerate(tiles):
            ok = True
            for a, n in enumerate((nT, nH, nW)):
                r = window[a] // 2
                lo = 0 if n <= 2 * r + 1 else min(max(tu[a] - r, 0), n - 1 - 2 * r)
                hi = n - 1 if n <= 2 * r + 1 else lo + 2 * r
                ok = ok and lo <= tv[a] <= hi
            assert keep[iu, iv] == ok
    assert np.array_equal(fo.tile_mask(g, window + (fo.EDGE_SHIFT,)), keep)


# ---- scales (Eq. 4) -----------------------------------------------------------------------
def test_scale_equals_float32_division_for_every_bf16_amax():
    bits = (np.arange(1, 0x7F80, dtype=np.uint32) << np.uint32(16))     # all positive finite bf16
    amax = bits.view(np.float32)
    want = amax / np.float32(448.0)
    got = fo._scale_from_amax(amax.astype(np.float64))
    assert got.dtype == np.float32 and np.array_equal(got.view(np.uint32), want.view(np.uint32))


def test_scale_closed_forms_and_exact_round_trip():
    g = fo.Geometry(1, 2, 4, 1, 2, 2)                                   # 2 tiles of 4 tokens
    d = 4
    vals = e4m3.decode(np.arange(0x7F, dtype=np.uint8))
    rng = np.random.default_rng(0)
    x = rng.choice(vals, size=(g.L_padded, d)) * rng.choice([-1, 1], size=(g.L_padded, d))
    x[0, 0] = 448.0
    x[g.TS, 1] = -448.0
    codes, s = fo.quantize_tiles(x, g)
    assert np.all(s == np.float32(1.0))                                  # amax 448 -> s = 1
    assert np.array_equal(e4m3.decode(codes), x)                         # representable -> exact
    for kexp in (-3, 0, 5):                                              # amax 7*2^k -> s = 2^k/64
        xs = x * (2.0 ** kexp) * (7.0 / 448.0)
        codes2, s2 = fo.quantize_tiles(xs, g)
        assert np.all(s2 == np.float32(2.0 ** kexp / 64.0))
        assert np.array_equal(codes2 & 0x7F, codes & 0x7F)
    z = np.zeros((g.L_padded, d))
    cz, sz = fo.quantize_tiles(z, g)
    assert np.all(sz == 1.0) and np.all(cz == 0)
    # per-channel variant: max over all tokens of the channel
    cc, sc = fo.quantize_channels(x)
    assert sc.shape == (d,) and np.array_equal(sc, (np.abs(x).max(axis=0) / 448).astype(np.float32))


def test_quantize_matches_brute_force_rational_rounding():
    g = SMALL
    q, _, _ = rand_qkv(11, (g.T, g.H, g.W), 8)
    codes, s = fo.quantize_tiles(fo.tile_order(q, g), g)
    deq = e4m3.decode(codes) * np.repeat(s.astype(np.float64), g.TS)[:, None]
    want, scales = brute.quantize_raster(q, (g.Tt, g.Th, g.Tw))
    assert np.array_equal(fo.tile_unorder(deq, g), want)
    nT, nH, nW = g.n_tiles_axis
    for (ut, uh, uw), sv in scales.items():
        assert s[(ut * nH + uh) * nW + uw] == sv
    # padded slots quantise to zero codes
    assert np.all((codes[~fo.valid_tokens(g)] & 0x7F) == 0)


# ---- schedule (Eq. 6) ---------------------------------------------------------------------
def test_schedule_three_regimes():
    D = 50
    picks = [fo.schedule_select(t, D, 0.2, 0.5) for t in range(1, D + 1)]
    assert picks == [0] * 10 + [1] * 15 + [2] * 25
    assert fo.schedule_select(1, 3, 0.34, 0.67) == 0 and fo.schedule_select(2, 3, 0.34, 0.67) == 1
    assert fo.schedule_select(3, 3, 0.34, 0.67) == 2
    with pytest.raises(AssertionError):
        fo.schedule_select(0, 50, 0.2, 0.5)


# ---- attention ----------------------------------------------------------------------------
def _dense_window(g):
    return tuple(2 * n - 1 for n in g.n_tiles_axis)


def test_dense_window_precision_off_is_textbook_softmax_attention():
    g = SMALL
    d = 16
    q, k, v = rand_qkv(1, (g.T, g.H, g.W), d)
    o = fo.attention(fo.tile_order(q, g), fo.tile_order(k, g), fo.tile_order(v, g), g,
                     _dense_window(g), prec=fo.PREC_BF16)
    o = fo.tile_unorder(o, g).reshape(-1, d)
    Q, K, V = q.reshape(-1, d), k.reshape(-1, d), v.reshape(-1, d)
    want = scipy.special.softmax(Q @ K.T / math.sqrt(d), axis=1) @ V
    assert np.max(np.abs(o - want)) <= 1e-12 * max(1.0, np.abs(want).max())
    # and as plain loops for three rows
    for i in (0, 17, 89):
        w = [math.exp(float(Q[i] @ K[j]) / math.sqrt(d)) for j in range(K.shape[0])]
        ref = sum(wj * V[j] for j, wj in enumerate(w)) / sum(w)
        assert np.max(np.abs(o[i] - ref)) <= 1e-12 * max(1.0, np.abs(ref).max())


@pytest.mark.parametrize("window", [(1, 3, 3), (3, 1, 1), (2, 2, 2)])
@pytest.mark.parametrize("fp8", [False, True])
def test_sparse_attention_matches_token_level_brute_force(window, fp8):
    g = SMALL
    d = 8
    q, k, v = rand_qkv(5 + fp8, (g.T, g.H, g.W), d)
    prec = fo.PREC_FP8 if fp8 else fo.PREC_BF16
    o = fo.attention(fo.tile_order(q, g), fo.tile_order(k, g), fo.tile_order(v, g), g, window,
                     prec=prec)
    o = fo.tile_unorder(o, g)
    want = brute.attention_raster(q, k, v, (g.Tt, g.Th, g.Tw), window, fp8)
    assert np.max(np.abs(o - want)) <= 1e-12 * np.abs(want).max()


def test_sub_tile_quantisation_groups_match_brute_force():
    """Quantisation granularity finer than the sparsity tile (g and W as separate
    hyper-parameters, Sec. 3.3): scales per sub-tile, window in whole tiles.  Pinned against the
    token-level brute force, where the sub-tiles are simply the grid cut into sub-tile boxes; the
    grid is ragged against the tile and against the sub-tile."""
    g = fo.Geometry(3, 5, 7, 2, 4, 4, 1, 2, 4)              # tile (2,4,4) in 4 sub-tiles of (1,2,4)
    assert g.NS == 4 and g.n_groups == g.M * 4
    d = 8
    q, k, v = rand_qkv(21, (g.T, g.H, g.W), d)
    # group bookkeeping: every sub-tile box of the raster grid is one group
    grp = fo.tile_unorder(fo.group_of_slot(g)[:, None].astype(np.float64), g)[..., 0]
    for t in range(g.T):
        for h in range(g.H):
            for w in range(g.W):
                same = grp == grp[t, h, w]
                box = np.zeros_like(same)
                box[t:t + 1, (h // 2) * 2:(h // 2) * 2 + 2, (w // 4) * 4:(w // 4) * 4 + 4] = True
                assert np.array_equal(same, box)
    # scales and codes against the brute force with the sub-tile as its quantisation box
    codes, s = fo.quantize_tiles(fo.tile_order(q, g), g)
    assert s.shape == (g.n_groups,)
    deq = e4m3.decode(codes) * s.astype(np.float64)[fo.group_of_slot(g)][:, None]
    want, _ = brute.quantize_raster(q, (1, 2, 4))
    assert np.array_equal(fo.tile_unorder(deq, g), want)
    coarse = fo.Geometry(3, 5, 7, 2, 4, 4)
    assert not np.array_equal(fo.quantize_tiles(fo.tile_order(q, coarse), coarse)[0], codes)
    for window in [(1, 3, 3), (3, 1, 1)]:
        o = fo.attention(fo.tile_order(q, g), fo.tile_order(k, g), fo.tile_order(v, g), g, window)
        want = brute.attention_raster(q, k, v, (2, 4, 4), window, True, qtile=(1, 2, 4))
        assert np.max(np.abs(fo.tile_unorder(o, g) - want)) <= 1e-12 * np.abs(want).max()
    # a sub-tile equal to the tile is the unified granularity, bit for bit
    same = fo.Geometry(3, 5, 7, 2, 4, 4, 2, 4, 4)
    a = fo.attention(fo.tile_order(q, same), fo.tile_order(k, same), fo.tile_order(v, same), same, (1, 3, 3))
    b = fo.attention(fo.tile_order(q, coarse), fo.tile_order(k, coarse), fo.tile_order(v, coarse), coarse, (1, 3, 3))
    assert np.array_equal(a, b)
    with pytest.raises(AssertionError):
        fo.Geometry(3, 5, 7, 2, 4, 4, 1, 3, 4)                # a sub-tile must divide the tile


def test_channelwise_v_matches_brute_force():
    g = fo.Geometry(2, 3, 4, 1, 2, 2)
    d = 4
    q, k, v = rand_qkv(9, (g.T, g.H, g.W), d)
    o = fo.attention(fo.tile_order(q, g), fo.tile_order(k, g), fo.tile_order(v, g), g, (3, 1, 3),
                     prec=fo.PREC_FP8, vscale=fo.VSCALE_CHANNEL)
    want = brute.attention_raster(q, k, v, (g.Tt, g.Th, g.Tw), (3, 1, 3), True, v_per_channel=True)
    assert np.max(np.abs(fo.tile_unorder(o, g) - want)) <= 1e-12 * np.abs(want).max()


def test_zero_queries_give_window_mean_of_dequantised_values():
    g = SMALL
    d = 8
    window = (1, 3, 1)
    _, k, v = rand_qkv(21, (g.T, g.H, g.W), d)
    q = np.zeros_like(k)
    o = fo.tile_unorder(fo.attention(fo.tile_order(q, g), fo.tile_order(k, g), fo.tile_order(v, g),
                                     g, window, prec=fo.PREC_FP8), g)
    vdq, _ = brute.quantize_raster(v, (g.Tt, g.Th, g.Tw))
    # S' = 0, m = 0, P = 1 exactly: O = plain mean of dequantised V over the real tokens of W(u)
    for (t, h, w) in [(0, 0, 0), (2, 4, 5), (1, 2, 3), (2, 0, 4)]:
        tu = brute.tile_of(t, h, w, (g.Tt, g.Th, g.Tw))
        acc, n = np.zeros(d), 0
        for tt in range(g.T):
            for hh in range(g.H):
                for ww in range(g.W):
                    if brute.in_window(tu, brute.tile_of(tt, hh, ww, (g.Tt, g.Th, g.Tw)), window):
                        acc += vdq[tt, hh, ww]
                        n += 1
        assert np.max(np.abs(o[t, h, w] - acc / n)) <= 1e-13


def test_padded_slots_contribute_nothing():
    g = SMALL
    d = 8
    q, k, v = rand_qkv(31, (g.T, g.H, g.W), d)
    qt, kt, vt = (fo.tile_order(a, g) for a in (q, k, v))
    pad = ~fo.valid_tokens(g)
    for prec in (fo.PREC_BF16, fo.PREC_FP8):
        base = fo.attention(qt, kt, vt, g, (3, 3, 3), prec=prec)
        kt2, vt2, qt2 = kt.copy(), vt.copy(), qt.copy()
        if prec == fo.PREC_BF16:
            kt2[pad] = 1e30
            vt2[pad] = -1e30
            qt2[pad] = 7.0
        else:
            # after quantisation-stage zeroing garbage may not raise the tile amax: keep it small
            kt2[pad] = 2.0 ** -20
            vt2[pad] = -(2.0 ** -20)
            qt2[pad] = 2.0 ** -20
        other = fo.attention(qt2, kt2, vt2, g, (3, 3, 3), prec=prec)
        assert np.array_equal(base[~pad], other[~pad])
        assert np.all(other[pad] == 0) and np.all(base[pad] == 0)
    # amax is unchanged by the zero padding
    s_pad = fo.tile_scales(kt, g)
    nT, nH, nW = g.n_tiles_axis
    blk = k[0:2, 4:5, 4:6]
    assert s_pad[(0 * nH + 2) * nW + 1] == np.float32(np.abs(blk).max() / 448.0)


def test_softmax_mass():
    g = fo.Geometry(2, 4, 4, 1, 2, 2)
    d = 8
    q, k, v = rand_qkv(41, (g.T, g.H, g.W), d, outlier=False)
    ones = np.ones_like(v)
    qt, kt, vt = (fo.tile_order(a, g) for a in (q, k, ones))
    o = fo.attention(qt, kt, vt, g, (3, 3, 3), prec=fo.PREC_BF16)
    assert np.max(np.abs(o - 1.0)) <= 1e-15 * 8          # rows of P/l sum to one
    # FP8: V = 1 is representable (amax 1 -> s = 1/448, code 448) so O = sum(P_hat)/l, within the
    # e4m3 relative rounding bound 2^-4 plus the mass flushed below the smallest subnormal
    o8 = fo.attention(qt, kt, vt, g, (3, 3, 3), prec=fo.PREC_FP8)
    assert np.max(np.abs(o8 - 1.0)) <= 2.0 ** -4 + g.L_real * 2.0 ** -10 / 448 / 0.5
    assert np.max(np.abs(o8 - 1.0)) > 0


def test_translation_equivariance_in_the_interior():
    g = fo.Geometry(6, 8, 8, 1, 2, 2)
    d = 8
    window = (3, 3, 3)
    q, k, v = rand_qkv(51, (g.T, g.H, g.W), d)
    o = fo.tile_unorder(fo.attention(*(fo.tile_order(a, g) for a in (q, k, v)), g, window), g)
    sh = (1, 2, 2)                                           # one tile along every axis
    q2, k2, v2 = (np.roll(a, sh, axis=(0, 1, 2)) for a in (q, k, v))
    o2 = fo.tile_unorder(fo.attention(*(fo.tile_order(a, g) for a in (q2, k2, v2)), g, window), g)
    # tiles whose whole window lies inside the grid before and after the shift
    inner = (slice(1, 4), slice(2, 4), slice(2, 4))
    moved = (slice(2, 5), slice(4, 6), slice(4, 6))
    assert np.array_equal(o[inner], o2[moved])


def test_hand_sized_case_with_subnormal_p():
    """One key tile, three keys, d = 2: every step is recomputed with scalar Python and rational
    FP8 rounding.  For query 0 the three P values land in the three regimes of the 1/448-scaled
    e4m3 grid: normal range, flushed to zero, and subnormal range (below 2^-6)."""
    g = fo.Geometry(1, 1, 3, 1, 1, 3)
    q = np.array([[[[4.0, 0.0], [0.5, 1.0], [-3.0, 2.0]]]])
    k = np.array([[[[6.0, 1.0], [-6.0, 0.5], [2.0, -2.0]]]])
    v = np.array([[[[1.0, -2.0], [3.0, 0.5], [-1.5, 8.0]]]])
    assert q.shape == (1, 1, 3, 2)
    o = fo.tile_unorder(fo.attention(fo.tile_order(q, g), fo.tile_order(k, g), fo.tile_order(v, g),
                                     g, (1, 1, 1)), g)
    want = brute.attention_raster(q, k, v, (1, 1, 3), (1, 1, 1), True)
    assert np.max(np.abs(o - want)) <= 1e-14
    qd, _ = brute.quantize_raster(q, (1, 1, 3))
    kd, _ = brute.quantize_raster(k, (1, 1, 3))
    vd, _ = brute.quantize_raster(v, (1, 1, 3))
    s = [float(qd[0, 0, 0] @ kd[0, 0, j]) / math.sqrt(2) * math.log2(math.e) for j in range(3)]
    m = math.ceil(max(s))
    y = [448.0 * 2.0 ** (x - m) for x in s]
    assert 224 < y[0] <= 448 and y[1] < 2.0 ** -10 and 2.0 ** -10 < y[2] < 2.0 ** -6
    yq = e4m3.round_to_e4m3(np.array(y))
    assert yq[1] == 0.0 and (yq[2] * 512) == round(y[2] * 512) and yq[0] % 16 == 0
    l = sum(2.0 ** (x - m) for x in s)
    ref = (yq[0] * vd[0, 0, 0] + yq[2] * vd[0, 0, 2]) / 448.0 / l
    assert np.max(np.abs(o[0, 0, 0] - ref)) <= 1e-14


def test_parts_are_consistent_with_the_output():
    g = fo.Geometry(1, 2, 4, 1, 2, 4)
    d = 8
    q, k, v = rand_qkv(61, (g.T, g.H, g.W), d, outlier=False)
    o, parts = fo.attention(*(fo.tile_order(a, g) for a in (q, k, v)), g, (1, 1, 1), return_parts=True)
    assert len(parts) == g.M
    pt = parts[0]
    assert np.array_equal(o[:g.TS], (pt["ph"] @ pt["v"]) / pt["l"][:, None])
    assert np.array_equal(pt["S"], pt["raw"] * pt["pair_scale"])
    assert np.all(pt["p"] <= 1.0) and np.all(pt["p"].max(axis=1) > 0.5)
    assert np.all(np.abs(pt["ph"] - pt["p"]) <= np.maximum(pt["p"] * 2.0 ** -4, 2.0 ** -10 / 448))
