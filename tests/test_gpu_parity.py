"""GPU parity: every step of the HIP path, called through the C ABI, against the CPU oracle."""
import dataclasses
import sys

import numpy as np
import pytest

from oracle import e4m3
from oracle import fps_oracle as fo
from paper_2506_04648_amd import fps, synth
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def tiny():
    return gu.GpuRun(synth.TINY)


# ---- layout and quantisation: bit exact -----------------------------------------------------
@pytest.mark.parametrize("grid,tile", [((4, 16, 16), (2, 4, 4)), ((3, 5, 6), (2, 4, 4)),
                                       ((2, 9, 20), (1, 8, 16)), ((3, 7, 9), (2, 4, 16)),
                                       ((3, 13, 20), (2, 8, 16)), ((7, 9, 10), (6, 8, 8)),
                                       ((5, 7, 9), (3, 4, 4)), ((2, 9, 20), (1, 7, 15)),
                                       ((3, 5, 6), (2, 8, 4))])
def test_tile_order_roundtrip_bit_exact(grid, tile):
    import torch
    say("tile_order", grid, tile)
    w = dataclasses.replace(synth.TINY, grid=grid, tile=tile, heads=3)
    run = gu.GpuRun(w)
    for a, t in zip(run.qkv, run.tiled):
        want = fo.tile_order(a, run.g)
        got = t[0].float().cpu().numpy()
        assert np.array_equal(got[:, run.slots], want)
        assert np.all(got[:, run.pad_slots()] == 0)
        back = fps.tile_unorder(run.shape, t)
        assert np.array_equal(back[0].float().cpu().numpy(), a)
        back32 = fps.tile_unorder(run.shape, t.float().contiguous())
        assert np.array_equal(back32[0].cpu().numpy(), a)


def _check_quantize(run, heads_slots, label):
    g = run.g
    for role, (xq, sc) in enumerate(run.quantize()):
        codes = fps.debug_unpack_q8(run.shape, xq, role)[0].cpu().numpy()
        sc = sc[0].cpu().numpy()
        for hs in heads_slots:
            x = fo.tile_order(run.qkv[role][hs].astype(np.float64), g)
            wc, ws = fo.quantize_tiles(x, g)
            assert np.array_equal(sc[hs].view(np.uint32), ws.view(np.uint32)), (label, role, hs)
            got = codes[hs][run.slots]
            zero_sign = ((got ^ wc) == 0x80) & ((wc & 0x7F) == 0)
            mism = (got != wc) & ~zero_sign
            assert int(mism.sum()) == 0, (label, role, hs, int(mism.sum()))
            assert np.all((codes[hs][run.pad_slots()] & 0x7F) == 0)
        assert not np.any((codes & 0x7F) == 0x7F)


def test_quantize_tiny_bit_exact(tiny):
    say("quantize tiny")
    _check_quantize(tiny, range(2), "tiny")


def test_quantize_ragged_128_token_tiles_bit_exact():
    say("quantize ragged 128")
    w = dataclasses.replace(synth.TINY, grid=(2, 13, 40), tile=(1, 8, 16), heads=2, n_outlier=3)
    _check_quantize(gu.GpuRun(w), range(2), "ragged128")


@pytest.mark.parametrize("grid,tile", [((3, 13, 20), (2, 8, 16)),      # 256 tokens; last T tile half empty
                                       ((7, 9, 10), (6, 8, 8)),         # 384 tokens, ragged on every axis
                                       ((5, 16, 20), (4, 16, 16)),      # 1024 tokens
                                       ((5, 7, 9), (3, 4, 4)),          # 48 tokens in two 32-slot blocks
                                       ((2, 9, 20), (1, 7, 15)),        # 105 tokens in one 128-slot block
                                       ((13, 17, 20), (12, 16, 16)),    # 3072 tokens, 24 blocks
                                       ((25, 5, 6), (24, 32, 32))])     # 24576 tokens, 192 blocks, mostly padding
def test_quantize_tiles_of_several_blocks_bit_exact(grid, tile):
    """One scale per TILE although the kernels work on 128-token blocks (tile amax pre-pass)."""
    say("quantize multi-block", grid, tile)
    w = dataclasses.replace(synth.TINY, grid=grid, tile=tile, heads=2, n_outlier=3, config_id=15)
    run = gu.GpuRun(w)
    assert run.quantize()[0][1].shape[-1] == run.g.M
    _check_quantize(run, range(2), f"multi-block {tile}")


SUB_TILE_CASES = [
    ((3, 13, 20), (2, 8, 16), (1, 8, 16)),      # sub-tile = one 128-slot block, 2 per tile
    ((7, 9, 10), (6, 8, 8), (2, 8, 8)),         # 3 sub-tiles of 128 tokens
    ((5, 9, 18), (4, 8, 8), (2, 4, 8)),         # 4 sub-tiles of 64 tokens: two 32-slot blocks each
    ((3, 5, 6), (2, 4, 4), (1, 2, 4)),          # 4 sub-tiles of 8 tokens in a 32-slot block each
    ((5, 16, 20), (4, 16, 16), (2, 8, 16)),     # 8 sub-tiles of 256 tokens (two 128-slot blocks each)
    ((3, 9, 20), (2, 7, 15), (1, 7, 5)),        # 6 sub-tiles of 35 tokens in two 32-slot blocks each
]


@pytest.mark.parametrize("grid,tile,qtile", SUB_TILE_CASES)
def test_quantisation_sub_tiles_layout_and_codes_bit_exact(grid, tile, qtile):
    """Scales per sub-tile of the sparsity tile: tile order round trip, scales and codes."""
    import torch
    say("sub-tile quantise", grid, tile, qtile)
    w = dataclasses.replace(synth.TINY, grid=grid, tile=tile, heads=2, n_outlier=3, config_id=19)
    run = gu.GpuRun(w, qtile=qtile)
    for a, t in zip(run.qkv, run.tiled):
        got = t[0].float().cpu().numpy()
        assert np.array_equal(got[:, run.slots], fo.tile_order(a, run.g))
        assert np.all(got[:, run.pad_slots()] == 0)
        assert np.array_equal(fps.tile_unorder(run.shape, t)[0].float().cpu().numpy(), a)
    assert run.quantize()[0][1].shape[-1] == run.g.n_groups
    _check_quantize(run, range(2), f"sub-tile {tile} {qtile}")
    p16 = run.pack_bf16()
    for role in range(3):                                   # fused raster entries == tiled entries
        xq, sc = fps.quantize_tiles(run.shape, run.raster[role], role, raster=True)
        assert torch.equal(xq, run.q8[role][0]) and torch.equal(sc, run.q8[role][1])
        xp, vs = fps.pack_tiles_bf16(run.shape, run.raster[role], role, raster=True)
        assert torch.equal(xp, p16[role][0])
        assert (vs is None and p16[role][1] is None) or torch.equal(vs, p16[role][1])


@pytest.mark.parametrize("prec", [fps.PREC_FP8, fps.PREC_BF16])
@pytest.mark.parametrize("grid,tile,qtile", SUB_TILE_CASES)
def test_attention_with_quantisation_sub_tiles(prec, grid, tile, qtile):
    import torch
    say("sub-tile attention", prec, grid, tile, qtile)
    window = (3, 3, 3)
    w = dataclasses.replace(synth.TINY, grid=grid, tile=tile, window=window, heads=2, n_outlier=3,
                            config_id=20)
    run = gu.GpuRun(w, qtile=qtile)
    out, vis = run.attn(prec, visited=True)
    assert np.array_equal(vis.cpu().numpy().astype(bool), fo.tile_mask(run.g, window))
    for h in range(2):
        st = gu.compare_head(run, out, h, prec, window)
        say("  head", h, st)
        gu.assert_parity(st, f"{grid} {tile} {qtile} head {h}")
    raster = run.attn(prec, raster_out=True)
    assert torch.equal(raster, fps.tile_unorder(run.shape, out))
    if prec == fps.PREC_FP8:                                # per-channel V with sub-tile Q/K scales
        out = run.attn(prec, vscale=fps.VSCALE_CHANNEL)
        st = gu.compare_head(run, out, 0, prec, window, vscale=fps.VSCALE_CHANNEL)
        say("  per-channel V", st)
        gu.assert_parity(st, f"{grid} {tile} {qtile} per-channel V")


def test_quantize_special_values():
    """Ties of the exact quotient, e4m3-representable inputs, all-zero tiles, amax = 448."""
    import torch
    say("quantize special")
    g = fo.Geometry(1, 8, 32, 1, 8, 16)                      # two tiles of 128 tokens
    shape = fps.make_shape(1, (1, 8, 32), (1, 8, 16))
    rng = np.random.default_rng(0)
    vals = e4m3.decode(np.arange(0x7F, dtype=np.uint8))
    mids = 0.5 * (vals[:-1] + vals[1:])
    x = np.zeros((g.L_padded, 128))
    # tile 0: amax 448 -> s = 1: representable values and every midpoint, both signs
    pool = np.concatenate([vals, mids, -vals, -mids])
    pool = pool[np.abs(pool) <= 448]
    t0 = rng.choice(pool, size=(128, 128))
    t0[0, 0] = 448.0
    # tile 1: amax = 7 * c with c = 29 -> many mathematically exact midpoints x*448/amax
    amax = 7.0 * 29.0 / 64.0
    cands = np.array([(2 * n + 1) * 29.0 / 64.0 * 2.0 ** -k for n in range(16) for k in range(0, 9)])
    cands = cands[(cands <= amax)]
    t1 = rng.choice(np.concatenate([cands, -cands]), size=(128, 128))
    t1[5, 7] = amax
    x[:128], x[128:] = t0, t1
    xb = synth.round_to_bf16(x.astype(np.float32)).astype(np.float64)
    tiled = gu.to_device_bf16(xb.astype(np.float32)[None, None])
    for role in (0, 1, 2):
        xq, sc = fps.quantize_tiles(shape, tiled, role)
        codes = fps.debug_unpack_q8(shape, xq, role)[0, 0].cpu().numpy()
        wc, ws = fo.quantize_tiles(xb, g)
        assert np.array_equal(sc[0, 0].cpu().numpy(), ws)
        zero_sign = ((codes ^ wc) == 0x80) & ((wc & 0x7F) == 0)
        assert int(((codes != wc) & ~zero_sign).sum()) == 0, role
    z = torch.zeros((1, 1, g.L_padded, 128), dtype=torch.bfloat16, device="cuda:0")
    xq, sc = fps.quantize_tiles(shape, z, 1)
    assert torch.all(sc == 1.0) and torch.all(xq == 0)


# ---- the matrix instruction's accumulation accuracy -------------------------------------------
def test_score_accumulation_error_model(tiny):
    """Raw E4M3 scores of single tile pairs against the exact integer dot products: the layout is
    right (errors are tiny, not O(1)) and the hardware's accumulation error stays inside the bound
    the parity comparator assumes when it decides which P roundings are ambiguous."""
    say("score accumulation")
    tiny.quantize()
    worst = 0.0
    for h, u, v in [(0, 0, 0), (0, 5, 6), (1, 31, 27), (1, 12, 12), (0, 17, 21), (1, 3, 7)]:
        r, got, exact = gu.score_error_ratio(tiny, h, u, v)
        worst = max(worst, r)
        assert np.max(np.abs(got - exact)) <= 1e-3 * np.max(np.abs(exact))
    say("  tiny worst |dS| / sum|qk| = %.3e (bound %.3e)" % (worst, gu.ACC_EPS))
    assert worst <= gu.ACC_EPS
    w = dataclasses.replace(synth.TINY, grid=(2, 16, 32), tile=(1, 8, 16), heads=2, n_outlier=3,
                            config_id=11)
    run = gu.GpuRun(w)
    run.quantize()
    worst = 0.0
    for h, u, v in [(0, 0, 0), (0, 1, 2), (1, 7, 3), (1, 5, 5), (0, 6, 1)]:
        r, got, exact = gu.score_error_ratio(run, h, u, v)
        worst = max(worst, r)
    say("  128-token tiles worst |dS| / sum|qk| = %.3e" % worst)
    assert worst <= gu.ACC_EPS


def test_score_accumulation_bound_on_adversarial_codes():
    """Code patterns chosen to stress the matrix instruction's adder: a product of 448*448 beside
    127 products of 1*1 (the hardware drops the seven ones that share the large product's group of
    eight: the error is 7, not 127), cancelling large products over a small residue, uniformly
    random codes of the whole format, random powers of two over 15 binades.  All stay inside the
    accumulation bound the accepted set is built on."""
    say("adversarial codes")
    vals = e4m3.decode(np.arange(256, dtype=np.uint8))
    finite = vals[np.isfinite(vals)]
    rng = np.random.default_rng(7)

    def ratio(q, k, tile):
        w = dataclasses.replace(synth.TINY, grid=tile, tile=tile, heads=1, window=(1, 1, 1), config_id=23)
        run = gu.GpuRun(w, qkv=[a[None].astype(np.float32) for a in (q, k, np.zeros_like(q))])
        run.quantize()
        r, got, exact = gu.score_error_ratio(run, 0, 0, 0)
        return r / gu.ACC_EPS, float(np.max(np.abs(got - exact)))

    for tile in [(1, 8, 16), (2, 4, 4)]:                     # 128-slot and 32-slot blocks
        shp = tile + (128,)
        q = np.ones(shp)
        q[..., 0] = 448.0
        r, err = ratio(q, q.copy(), tile)
        say(f"  {tile} one dominant product: {r:.3f} of the bound, |err| {err:g}")
        assert r <= 1.0 and err <= 8.0
        q, k = np.ones(shp), np.ones(shp)
        q[..., 0] = q[..., 1] = k[..., 0] = 448.0
        k[..., 1] = -448.0
        r, err = ratio(q, k, tile)
        say(f"  {tile} cancelling pair: {r:.3f} of the bound, |err| {err:g}")
        assert r <= 1.0
        q, k = rng.choice(finite, shp), rng.choice(finite, shp)
        q[0, 0, 0, 0] = k[0, 0, 0, 0] = 448.0                # the tile scale is exactly 1
        r, err = ratio(q, k, tile)
        say(f"  {tile} uniformly random codes: {r:.3f} of the bound")
        assert r <= 1.0
        q = 2.0 ** rng.integers(-6, 9, shp) * rng.choice([-1.0, 1.0], shp)
        k = 2.0 ** rng.integers(-6, 9, shp) * rng.choice([-1.0, 1.0], shp)
        q[0, 0, 0, 0] = k[0, 0, 0, 0] = 448.0
        r, err = ratio(q, k, tile)
        say(f"  {tile} random powers of two: {r:.3f} of the bound")
        assert r <= 1.0


# ---- attention -------------------------------------------------------------------------------
def test_attention_tiny_fp8_full(tiny):
    say("attention tiny fp8")
    out, vis = tiny.attn(fps.PREC_FP8, visited=True)
    mask = fo.tile_mask(tiny.g, tiny.w.window)
    assert np.array_equal(vis.cpu().numpy().astype(bool), mask) and int(mask.sum()) == 200
    for h in range(2):
        st = gu.compare_head(tiny, out, h, fps.PREC_FP8, tiny.w.window)
        say("  head", h, st)
        gu.assert_parity(st, f"tiny fp8 head {h}")


@pytest.mark.parametrize("window", [(1, 3, 3), (3, 7, 7), (1, 1, 1), (2, 2, 2)])
def test_attention_tiny_bf16(tiny, window):
    say("attention tiny bf16", window)
    out, vis = tiny.attn(fps.PREC_BF16, window=window, visited=True)
    assert np.array_equal(vis.cpu().numpy().astype(bool), fo.tile_mask(tiny.g, window))
    for h in range(2):
        st = gu.compare_head(tiny, out, h, fps.PREC_BF16, window)
        say("  head", h, st)
        gu.assert_parity(st, f"tiny bf16 head {h}")


@pytest.mark.parametrize("window", [(3, 7, 7), (1, 1, 1), (2, 4, 6)])
def test_attention_tiny_fp8_windows(tiny, window):
    say("attention tiny fp8 window", window)
    out, vis = tiny.attn(fps.PREC_FP8, window=window, visited=True)
    assert np.array_equal(vis.cpu().numpy().astype(bool), fo.tile_mask(tiny.g, window))
    st = gu.compare_head(tiny, out, 1, fps.PREC_FP8, window)
    say("  ", st)
    gu.assert_parity(st, f"tiny fp8 {window}")


@pytest.mark.parametrize("prec", [fps.PREC_FP8, fps.PREC_BF16])
@pytest.mark.parametrize("grid,tile,window", [
    ((3, 5, 6), (2, 4, 4), (3, 3, 3)),          # ragged on every axis, 32-token tiles
    ((2, 13, 40), (1, 8, 16), (3, 3, 3)),       # ragged 128-token tiles, several tiles per axis
    ((1, 8, 16), (1, 8, 16), (1, 1, 1)),        # a single tile
    ((1, 3, 5), (1, 8, 16), (5, 5, 5)),         # a single, mostly padded tile
    ((5, 8, 16), (1, 8, 16), (2, 1, 1)),        # temporal-only window, even size
    ((3, 13, 20), (2, 8, 16), (3, 3, 3)),       # 256-token tiles (2 blocks); one key block all padding
    ((7, 9, 10), (6, 8, 8), (3, 1, 3)),         # 384-token tiles (3 blocks), ragged on every axis
    ((5, 16, 20), (4, 16, 16), (3, 1, 1)),      # 1024-token tiles (8 blocks)
    ((5, 7, 9), (3, 4, 4), (3, 3, 3)),          # 48-token tiles: two 32-slot blocks, 16 slots of padding
    ((3, 5, 12), (2, 8, 4), (3, 1, 3)),         # 64-token tiles: two 32-slot blocks
    ((2, 9, 20), (1, 7, 15), (3, 3, 3)),        # 105-token tiles in one 128-slot block
    ((13, 17, 20), (12, 16, 16), (3, 3, 3)),    # 3072-token tiles (24 blocks); skipped padding-only blocks
])
def test_attention_small_shapes(prec, grid, tile, window):
    say("attention small", prec, grid, tile, window)
    w = dataclasses.replace(synth.TINY, grid=grid, tile=tile, window=window, heads=2, n_outlier=3,
                            config_id=7)
    run = gu.GpuRun(w)
    out, vis = run.attn(prec, visited=True)
    assert np.array_equal(vis.cpu().numpy().astype(bool), fo.tile_mask(run.g, window))
    for h in range(2):
        st = gu.compare_head(run, out, h, prec, window)
        say("  head", h, st)
        gu.assert_parity(st, f"{grid} {tile} {window} head {h}")


@pytest.mark.parametrize("grid,tile,window", [((4, 16, 16), (2, 4, 4), (1, 3, 3)),
                                              ((2, 13, 40), (1, 8, 16), (3, 3, 3)),
                                              ((3, 13, 20), (2, 8, 16), (3, 3, 3))])
def test_per_channel_v_scales(grid, tile, window):
    """The paper's own V quantisation (Sec. 3.2): one scale per channel over all tokens."""
    import torch
    say("per-channel V", grid, tile)
    w = dataclasses.replace(synth.TINY, grid=grid, tile=tile, window=window, heads=2, n_outlier=3,
                            config_id=13)
    run = gu.GpuRun(w)
    xq, sc = fps.quantize_tiles(run.shape, run.tiled[2], fps.ROLE_V, vscale=fps.VSCALE_CHANNEL)
    xq_r, sc_r = fps.quantize_tiles(run.shape, run.raster[2], fps.ROLE_V, vscale=fps.VSCALE_CHANNEL,
                                    raster=True)
    assert torch.equal(xq, xq_r) and torch.equal(sc, sc_r) and sc.shape == (1, 2, 128)
    codes = fps.debug_unpack_q8(run.shape, xq, fps.ROLE_V)[0].cpu().numpy()
    for h in range(2):
        wc, ws = fo.quantize_channels(fo.tile_order(run.qkv[2][h].astype(np.float64), run.g))
        assert np.array_equal(sc[0, h].cpu().numpy(), ws)
        got = codes[h][run.slots]
        zero_sign = ((got ^ wc) == 0x80) & ((wc & 0x7F) == 0)
        assert int(((got != wc) & ~zero_sign).sum()) == 0
    out = run.attn(fps.PREC_FP8, vscale=fps.VSCALE_CHANNEL)
    for h in range(2):
        st = gu.compare_head(run, out, h, fps.PREC_FP8, window, vscale=fps.VSCALE_CHANNEL)
        say("  head", h, st)
        gu.assert_parity(st, f"per-channel V head {h}")


@pytest.mark.parametrize("prec", [fps.PREC_FP8, fps.PREC_BF16])
def test_shifted_window_edge_rule(prec):
    say("shifted window", prec)
    w = dataclasses.replace(synth.TINY, grid=(5, 13, 40), tile=(1, 8, 16), window=(3, 1, 3), heads=1,
                            n_outlier=3, config_id=14)
    run = gu.GpuRun(w)
    win = w.window + (fps.EDGE_SHIFT,)
    out, vis = run.attn(prec, window=win, visited=True)
    mask = fo.tile_mask(run.g, win)
    assert np.array_equal(vis.cpu().numpy().astype(bool), mask)
    assert np.all(mask.sum(axis=1) == 3 * 1 * 3)
    st = gu.compare_head(run, out, 0, prec, win)
    say("  ", st)
    gu.assert_parity(st, "shifted window")


def test_shared_outlier_channels_stress():
    """Q and K share their outlier channels: the score spread is ~10x larger (|S'| ~ 100, rows
    close to one-hot), outside the input distribution the tolerances are stated for.  The error of
    the hardware's FP8 accumulation (about 2^-14 of sum|q_c k_c|) then moves the softmax weights
    themselves by a few 1e-3, so only looser bounds are asserted here: finite, padded rows zero,
    max excess <= 1e-1 RMS, mean <= 5e-3 RMS."""
    say("attention stress")
    w = dataclasses.replace(synth.TINY, grid=(2, 8, 32), tile=(1, 8, 16), window=(3, 1, 3), heads=1,
                            config_id=8)
    q, k, v = synth.qkv_raster(w)
    q_out = q.reshape(-1, 128).std(axis=0) > 4
    k_out = k.reshape(-1, 128).std(axis=0) > 4
    k = k.copy()
    k[..., k_out] /= 8                                     # undo K's own outlier channels ...
    k[..., q_out] *= 8                                     # ... and put them where Q has its own
    k = synth.round_to_bf16(k)
    run = gu.GpuRun(w, qkv=(q, k, v))
    out = run.attn(fps.PREC_FP8)
    st = gu.compare_head(run, out, 0, fps.PREC_FP8, w.window)
    say("  ", st)
    assert st["finite"] and st["pad_rows_zero"]
    assert st["max_excess"] <= 1e-1 and st["mean_err"] <= 5e-3


def test_garbage_in_padded_slots_cannot_leak():
    import torch
    say("attention padded garbage")
    w = dataclasses.replace(synth.TINY, grid=(2, 13, 40), tile=(1, 8, 16), window=(3, 3, 3), heads=1,
                            n_outlier=3, config_id=9)
    run = gu.GpuRun(w)
    clean = run.attn(fps.PREC_FP8).clone()
    pad = torch.from_numpy(run.pad_slots()).to("cuda:0")
    for t in run.tiled:
        t[0, 0, pad] = 0.0078125                        # small: cannot raise any tile's amax
    del run.q8
    dirty = run.attn(fps.PREC_FP8)
    assert torch.equal(clean, dirty)


def test_bf16_output_is_rounded_fp32_output(tiny):
    import torch
    say("bf16 output")
    o32 = tiny.attn(fps.PREC_FP8, out_dtype=torch.float32)
    o16 = tiny.attn(fps.PREC_FP8, out_dtype=torch.bfloat16)
    assert torch.equal(o16, o32.to(torch.bfloat16))


@pytest.mark.parametrize("grid,tile", [((4, 16, 16), (2, 4, 4)), ((3, 5, 6), (2, 4, 4)),
                                       ((2, 13, 40), (1, 8, 16)), ((3, 13, 20), (2, 8, 16))])
def test_fused_raster_entry_points_match_the_unfused_path(grid, tile):
    """fps_quantize_raster == fps_tile_order + fps_quantize_tiles (bit for bit), and the raster
    output layout of fps_attn_fwd == fps_tile_unorder of the tiled output."""
    import torch
    say("fused raster", grid, tile)
    w = dataclasses.replace(synth.TINY, grid=grid, tile=tile, window=(3, 3, 3), heads=2, n_outlier=3,
                            config_id=12)
    run = gu.GpuRun(w)
    q8 = run.quantize()
    for role in range(3):
        xq, sc = fps.quantize_tiles(run.shape, run.raster[role], role, raster=True)
        assert torch.equal(xq, q8[role][0]) and torch.equal(sc, q8[role][1])
    p16 = run.pack_bf16()
    for role in range(3):
        xp, vs = fps.pack_tiles_bf16(run.shape, run.raster[role], role, raster=True)
        assert torch.equal(xp, p16[role][0])
        assert (vs is None and p16[role][1] is None) or torch.equal(vs, p16[role][1])
    for prec in (fps.PREC_FP8, fps.PREC_BF16):
        for dt in (torch.float32, torch.bfloat16):
            tiled = run.attn(prec, out_dtype=dt)
            raster = run.attn(prec, out_dtype=dt, raster_out=True)
            assert raster.shape == (1, 2) + tuple(grid) + (128,)
            assert torch.equal(raster, fps.tile_unorder(run.shape, tiled))


def test_two_runs_are_bit_identical_and_inputs_stay_untouched(tiny):
    import torch
    say("determinism")
    a = tiny.attn(fps.PREC_FP8).clone()
    before = [t.clone() for pair in tiny.q8 for t in pair] + [t.clone() for t in tiny.raster + tiny.tiled]
    b = tiny.attn(fps.PREC_FP8)
    assert torch.equal(a, b)
    fps.quantize_tiles(tiny.shape, tiny.raster[2], fps.ROLE_V, raster=True)
    fps.quantize_tiles(tiny.shape, tiny.tiled[0], fps.ROLE_Q)
    torch.cuda.synchronize()
    after = [t for pair in tiny.q8 for t in pair] + tiny.raster + tiny.tiled
    assert all(torch.equal(x, y) for x, y in zip(before, after))


def _random_case(rng):
    """A random small configuration: grid, tile, optional quantisation sub-tile, window, edge rule,
    precision, V scale granularity."""
    def divisors(n):
        return [d for d in range(1, n + 1) if n % d == 0]
    while True:
        tile = tuple(int(rng.choice(c)) for c in ([1, 2, 3, 4, 6], [1, 2, 4, 5, 8, 16], [2, 4, 5, 8, 16]))
        ts = tile[0] * tile[1] * tile[2]
        if not 8 <= ts <= 512:
            continue
        n_tiles = (int(rng.integers(1, 4)), int(rng.integers(1, 4)), int(rng.integers(1, 5)))
        grid = tuple(max(1, n * t - int(rng.integers(0, t))) for n, t in zip(n_tiles, tile))
        if grid[0] * grid[1] * grid[2] > 2600:
            continue
        qtile = None
        if rng.random() < 0.4:
            qtile = tuple(int(rng.choice(divisors(t))) for t in tile)
        window = tuple(int(rng.integers(1, 6)) for _ in range(3))
        if rng.random() < 0.3:
            window += (fps.EDGE_SHIFT,)
        prec = fps.PREC_FP8 if rng.random() < 0.7 else fps.PREC_BF16
        vscale = fps.VSCALE_CHANNEL if (prec == fps.PREC_FP8 and rng.random() < 0.3) else fps.VSCALE_TILE
        return grid, tile, qtile, window, prec, vscale


@pytest.mark.parametrize("seed", range(16))
def test_random_configurations(seed):
    """Seeded random shapes, tiles, sub-tiles, windows, edge rules and modes against the oracle."""
    rng = np.random.default_rng(1000 + seed)
    grid, tile, qtile, window, prec, vscale = _random_case(rng)
    say("random case", seed, grid, tile, qtile, window, prec, vscale)
    w = dataclasses.replace(synth.TINY, grid=grid, tile=tile, window=window[:3], heads=1, n_outlier=3,
                            config_id=100 + seed)
    run = gu.GpuRun(w, qtile=qtile)
    out, vis = run.attn(prec, window=window, visited=True, vscale=vscale)
    assert np.array_equal(vis.cpu().numpy().astype(bool), fo.tile_mask(run.g, window))
    if prec == fps.PREC_FP8:
        _check_quantize(run, [0], f"random {seed}") if vscale == fps.VSCALE_TILE else None
    st = gu.compare_head(run, out, 0, prec, window, vscale=vscale)
    say("  ", st)
    gu.assert_parity(st, f"random case {seed}: {grid} {tile} {qtile} {window} {prec} {vscale}")


def test_mfma_rate_kernel_runs():
    """The MFMA-only micro-benchmark kernel (yardstick of the roofline): every thread writes one
    finite value, and a thread's value grows linearly with the trip count (accumulator chains)."""
    import torch
    say("mfma rate")
    a = torch.full((8 * 256,), float("nan"), dtype=torch.float32, device="cuda:0")
    b = torch.full((8 * 256,), float("nan"), dtype=torch.float32, device="cuda:0")
    assert fps.debug_mfma_rate(8, 4, a) == 8 * 4 * 4 * 8 * 65536.0
    fps.debug_mfma_rate(8, 8, b)
    torch.cuda.synchronize()
    assert torch.isfinite(a).all() and torch.isfinite(b).all() and (a != 0).all()
    assert torch.equal(b, 2 * a)


def test_issue_mix_kernel_counts_shader_clocks():
    """The matrix/vector issue-mix micro-benchmark: every wave reports a clock count, and an
    MFMA-only loop of the E4M3 16x16x128 instruction takes its 8 passes (32 clocks) per instruction
    on a SIMD that holds one wave."""
    import torch
    say("issue mix")
    wgs, iters = 8, 200
    sink = torch.full((wgs * 256,), float("nan"), dtype=torch.float32, device="cuda:0")
    cyc = torch.zeros(wgs * 4, dtype=torch.int64, device="cuda:0")
    fps.debug_issue_mix(0, 0, 0, 1, wgs, iters, sink, cyc)
    torch.cuda.synchronize()
    per_mfma = cyc.double() / (iters * 8)
    assert torch.isfinite(sink).all() and (cyc > 0).all()
    assert 30.0 <= float(per_mfma.min()) and float(per_mfma.max()) <= 40.0, per_mfma
    for kind, nv, op in [(1, 4, 0), (2, 8, 1), (3, 16, 0)]:
        cyc.zero_()
        fps.debug_issue_mix(kind, nv, op, 2, wgs, iters, sink, cyc)
        torch.cuda.synchronize()
        assert (cyc > 0).all() and torch.isfinite(sink).all()
    with pytest.raises(fps.FpsError):
        fps.debug_issue_mix(0, 5, 0, 1, wgs, iters, sink, cyc)          # not one of the built group sizes


def test_batch_and_heads_are_interchangeable():
    """Tensors are indexed by b*heads + h: (B=2, heads=3) equals (B=1, heads=6) bit for bit."""
    import torch
    say("batch")
    w = dataclasses.replace(synth.TINY, grid=(2, 13, 40), tile=(1, 8, 16), window=(3, 3, 3), heads=6,
                            n_outlier=3, config_id=18)
    run = gu.GpuRun(w)
    flat = fps.make_shape(6, w.grid, w.tile, B=1)
    two = fps.make_shape(3, w.grid, w.tile, B=2)
    outs = []
    for sh, lead in ((flat, (1, 6)), (two, (2, 3))):
        x = [r.reshape(lead + r.shape[2:]) for r in run.raster]
        q8 = [fps.quantize_tiles(sh, x[i], i, raster=True) for i in range(3)]
        assert q8[0][1].shape == lead + (run.g.M,)
        o = fps.attn_fwd(sh, w.window, fps.PREC_FP8, q8[0][0], q8[1][0], q8[2][0], q8[0][1], q8[1][1],
                         q8[2][1], out_dtype=torch.float32, raster_out=True)
        assert o.shape == lead + tuple(w.grid) + (128,)
        outs.append(o.reshape(-1))
    torch.cuda.synchronize()
    assert torch.equal(outs[0], outs[1])


def test_side_stream_and_graph_replay(tiny):
    """The library launches on the stream it is given and allocates nothing, so the whole path
    (three fused quantise passes + attention) can run on a side stream and be captured into a HIP
    graph; every replay, with eager work and synchronisations in between, reproduces the eager
    result bit for bit."""
    import torch
    say("stream + graph")
    shape, w = tiny.shape, tiny.w
    M = tiny.g.M
    packed = [torch.empty(fps.packed_bytes(shape, fps.PREC_FP8), dtype=torch.uint8, device="cuda:0") for _ in range(3)]
    scales = [torch.empty((1, w.heads, M), dtype=torch.float32, device="cuda:0") for _ in range(3)]
    out = torch.empty((1, w.heads) + tuple(w.grid) + (128,), dtype=torch.float32, device="cuda:0")

    def path():
        for i in range(3):
            fps.quantize_tiles(shape, tiny.raster[i], i, out=packed[i], scales=scales[i], raster=True)
        fps.attn_fwd(shape, w.window, fps.PREC_FP8, packed[0], packed[1], packed[2], scales[0], scales[1],
                     scales[2], out=out, raster_out=True)

    path()
    torch.cuda.synchronize()
    want = out.clone()
    side = torch.cuda.Stream()                      # default priority
    side.wait_stream(torch.cuda.current_stream())
    out.zero_()
    with torch.cuda.stream(side):
        path()
    side.synchronize()
    assert torch.equal(out, want)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        path()
    for rep in range(4):
        out.fill_(float(rep))                        # eager work between the replays
        for p_ in packed:
            p_.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, want), rep


def test_calls_on_two_streams_at_once_do_not_disturb_each_other(tiny):
    """The library keeps no device state between calls: two different shapes driven from two
    streams at the same time give what each gives alone."""
    import torch
    say("two streams at once")
    other = gu.GpuRun(dataclasses.replace(synth.TINY, grid=(5, 13, 20), tile=(1, 8, 16), window=(3, 3, 3),
                                          heads=3, n_outlier=3, config_id=29))
    runs = [tiny, other]
    want = []
    for r in runs:
        r.quantize()
        want.append(r.attn(fps.PREC_FP8).clone())
    outs = [torch.empty_like(o) for o in want]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]          # default priority
    for st in streams:
        st.wait_stream(torch.cuda.current_stream())
    for rep in range(8):
        for r, o, st in zip(runs, outs, streams):
            with torch.cuda.stream(st):
                (q, sq), (k, sk), (v, sv) = r.q8
                fps.attn_fwd(r.shape, r.w.window, fps.PREC_FP8, q, k, v, sq, sk, sv, out=o)
    for st in streams:
        st.synchronize()
    for o, x in zip(outs, want):
        assert torch.equal(o, x)


def test_step_config_selects_regime(tiny):
    import torch
    say("step config")
    regimes = [(fps.PREC_BF16, (3, 7, 7)), (fps.PREC_FP8, (3, 3, 3)), (fps.PREC_FP8, (1, 3, 3))]
    for step, idx in ((1, 0), (20, 1), (50, 2)):
        cfg = fps.make_step_cfg(step, 50, 0.2, 0.5, regimes)
        prec, win = fps.schedule_select(cfg)
        assert (prec, win) == regimes[idx]
        want = tiny.attn(prec, window=win)
        got = tiny.attn(prec, window=(9, 9, 9), step=cfg)     # explicit window must be overridden
        assert torch.equal(want, got)


def test_largest_granularity_of_the_tile_size_ablation():
    """(24,32,32) tiles (Table 3's largest): 24576 slots per tile, 192 blocks; the comparator
    fetches the kernel's scores block pair by block pair."""
    say("24x32x32 tiles")
    w = dataclasses.replace(synth.TINY, grid=(25, 5, 6), tile=(24, 32, 32), window=(3, 1, 1), heads=1,
                            n_outlier=3, config_id=16)
    run = gu.GpuRun(w)
    assert run.tsp == 24576 and run.g.M == 2
    for prec in (fps.PREC_BF16, fps.PREC_FP8):
        out, vis = run.attn(prec, visited=True)
        assert np.array_equal(vis.cpu().numpy().astype(bool), fo.tile_mask(run.g, w.window))
        st = gu.compare_head(run, out, 0, prec, w.window)
        say("  ", prec, st)
        gu.assert_parity(st, f"24x32x32 prec {prec}")


def test_step_config_with_granularity_per_regime():
    """Eq. 6: every regime has its own tile granularity g(t) and window W(t).  The caller
    quantises with the tile of the step's regime; a call whose inputs have another tile is
    refused."""
    say("step config with g(t)")
    regimes = [(fps.PREC_FP8, (1, 1, 3), (6, 8, 8)),        # early: coarse tiles, sparse window
               (fps.PREC_FP8, (3, 3, 3), (1, 8, 16)),       # mid: fine tiles, dense window
               (fps.PREC_FP8, (1, 3, 3), (2, 8, 16))]       # late: in between
    runs = {}
    for step, idx in ((3, 0), (20, 1), (44, 2)):
        cfg = fps.make_step_cfg(step, 50, 0.2, 0.5, regimes)
        prec, win, tile = fps.schedule_select(cfg, with_tile=True)
        assert (prec, win, tile) == regimes[idx]
        w = dataclasses.replace(synth.TINY, grid=(7, 13, 20), tile=tile, window=win, heads=1,
                                n_outlier=3, config_id=17)
        run = runs[idx] = gu.GpuRun(w)
        out = run.attn(prec, window=(9, 9, 9), step=cfg)     # the explicit window is overridden
        st = gu.compare_head(run, out, 0, prec, win)
        say("  step", step, tile, win, st)
        gu.assert_parity(st, f"step {step}")
    with pytest.raises(fps.FpsError) as e:                   # inputs of the late regime at an early step
        runs[2].attn(fps.PREC_FP8, step=fps.make_step_cfg(3, 50, 0.2, 0.5, regimes))
    assert e.value.status == fps.FPS_ERR_INVALID_ARG
    # a regime may also fix the quantisation sub-tile: same sparsity tile, finer scales
    fine = [(fps.PREC_FP8, (1, 3, 3), (2, 8, 16), (1, 8, 16))] * 3
    cfg = fps.make_step_cfg(44, 50, 0.2, 0.5, fine)
    assert fps.schedule_select(cfg, with_tile=True) == fine[0]
    with pytest.raises(fps.FpsError):
        runs[2].attn(fps.PREC_FP8, step=cfg)                 # quantised per tile, regime wants per sub-tile
    w = dataclasses.replace(synth.TINY, grid=(7, 13, 20), tile=(2, 8, 16), window=(1, 3, 3), heads=1,
                            n_outlier=3, config_id=17)
    run = gu.GpuRun(w, qtile=(1, 8, 16))
    st = gu.compare_head(run, run.attn(fps.PREC_FP8, step=cfg), 0, fps.PREC_FP8, (1, 3, 3))
    say("  sub-tile regime", st)
    gu.assert_parity(st, "sub-tile regime")


# ---- full-size shapes, sampled against the oracle ---------------------------------------------
def _sampled_parity(w, prec, window, head_picks, seed, n_interior=2, run=None):
    run = run or gu.GpuRun(w)
    out, vis = run.attn(prec, window=window, visited=True)
    mask = fo.tile_mask(run.g, window)
    assert np.array_equal(vis.cpu().numpy().astype(bool), mask)
    rng = np.random.default_rng(seed)
    for h in head_picks:
        tiles = gu.sample_q_tiles(run.g, rng, n_interior)
        st = gu.compare_head(run, out, h, prec, window, q_tiles=tiles)
        say(f"  {w.name} head {h} tiles {len(tiles)}", st)
        gu.assert_parity(st, f"{w.name} head {h}")
    return run, int(mask.sum())


def test_wan_1_3b_480p_fp8_sampled():
    say("480p fp8")
    run, pairs = _sampled_parity(synth.WAN_1_3B_480P, fps.PREC_FP8, synth.WAN_1_3B_480P.window,
                                 [0, 5, 11], seed=1)
    assert pairs == 6100
    # scales of every head and codes of one head per tensor, bit exact
    for role, (xq, sc) in enumerate(run.q8):
        sc = sc[0].cpu().numpy()
        for h in range(run.w.heads):
            ws = fo.tile_scales(fo.tile_order(run.qkv[role][h], run.g), run.g)
            assert np.array_equal(sc[h], ws)
        h = (5, 0, 11)[role]
        codes = fps.debug_unpack_q8(run.shape, xq, role)[0, h].cpu().numpy()[run.slots]
        wc, _ = fo.quantize_tiles(fo.tile_order(run.qkv[role][h].astype(np.float64), run.g), run.g)
        zero_sign = ((codes ^ wc) == 0x80) & ((wc & 0x7F) == 0)
        assert int(((codes != wc) & ~zero_sign).sum()) == 0, (role, h)


def test_wan_1_3b_480p_bf16_sparse_sampled():
    say("480p bf16")
    _sampled_parity(synth.WAN_1_3B_480P, fps.PREC_BF16, (3, 3, 3), [3], seed=2, n_interior=1)


def test_wan_14b_720p_fp8_sampled_in_bench_configuration():
    say("720p fp8")
    w = synth.WAN_14B_720P
    run, pairs = _sampled_parity(w, fps.PREC_FP8, w.window, [0, 17, 39], seed=3, n_interior=1)
    assert pairs == 20592
    for role, (xq, sc) in enumerate(run.q8):
        sc = sc[0].cpu().numpy()
        for h in range(0, w.heads, 7):
            ws = fo.tile_scales(fo.tile_order(run.qkv[role][h], run.g), run.g)
            assert np.array_equal(sc[h], ws)


def test_wan_14b_720p_dense_references_and_schedule_windows_sampled():
    """The other launches bench.py times on the 720p grid: the dense window in both precisions (the
    reference points of the speed-up) and the two FP8 windows of the step-aware schedule."""
    w = synth.WAN_14B_720P
    run = gu.GpuRun(w)
    nT, nH, nW = run.g.n_tiles_axis
    dense = (2 * nT - 1, 2 * nH - 1, 2 * nW - 1)
    for prec, window, pairs, head in [(fps.PREC_FP8, dense, 396900, 8), (fps.PREC_BF16, dense, 396900, 23),
                                      (fps.PREC_FP8, (7, 5, 5), 61560, 31), (fps.PREC_FP8, (3, 3, 3), 12688, 4)]:
        say("720p", "fp8" if prec == fps.PREC_FP8 else "bf16", window)
        _, kept = _sampled_parity(w, prec, window, [head], seed=5, n_interior=1, run=run)
        assert kept == pairs


def test_tensors_beyond_4_gib_index_correctly():
    """Offsets are 64-bit in every kernel: in a batch whose raster, packed and output tensors all
    exceed 2^32 bytes, the last heads give bit for bit what the same heads give alone."""
    import torch
    say("tensors beyond 4 GiB")
    w = dataclasses.replace(synth.WAN_1_3B_480P, heads=4, config_id=23)
    small = gu.GpuRun(w)
    reps = 200
    big = fps.make_shape(w.heads * reps, w.grid, w.tile)
    assert fps.packed_bytes(big, fps.PREC_FP8) > 2 ** 32
    results = []
    for shape, rasters in ((small.shape, small.raster),
                           (big, [r.repeat(1, reps, 1, 1, 1, 1) for r in small.raster])):
        assert shape is small.shape or rasters[0].numel() * 2 > 2 ** 32
        q8 = [fps.quantize_tiles(shape, r, role, raster=True) for role, r in enumerate(rasters)]
        o8 = fps.attn_fwd(shape, w.window, fps.PREC_FP8, q8[0][0], q8[1][0], q8[2][0],
                          q8[0][1], q8[1][1], q8[2][1], out_dtype=torch.bfloat16, raster_out=True)
        p16 = [fps.pack_tiles_bf16(shape, r, role, raster=True) for role, r in enumerate(rasters)]
        o16 = fps.attn_fwd(shape, w.window, fps.PREC_BF16, p16[0][0], p16[1][0], p16[2][0],
                           None, None, p16[2][1], out_dtype=torch.bfloat16, raster_out=True)
        torch.cuda.synchronize()
        n = shape.heads
        keep = [t.view(n, -1)[-w.heads:].clone() for pair in q8 + p16 for t in pair if t is not None]
        keep += [o.view(torch.int16).view(n, -1)[-w.heads:].clone() for o in (o8, o16)]
        results.append(keep)
        del q8, p16, o8, o16, rasters
    for i, (a, b) in enumerate(zip(*results)):
        assert torch.equal(a, b), f"tensor {i} of the last heads differs"
    assert float(results[0][-2].view(torch.bfloat16).float().abs().max()) > 0
