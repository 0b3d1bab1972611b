"""CPU-only checks of the C-ABI library: it loads, exports what include/fps.h declares, and its
host logic (schedule, tile mask, argument validation) agrees with the oracle.  No kernel runs."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import fps_oracle as fo
from paper_2506_04648_amd import fps

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "fps.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(fps_[a-z0-9_]+)\s*\(", header))
    assert declared == set(fps.EXPORTS)
    L = fps.lib()
    for name in declared:
        assert getattr(L, name) is not None
    assert fps.last_error() is not None


def test_schedule_select_matches_oracle():
    regimes = [(fps.PREC_BF16, (41, 11, 9)), (fps.PREC_FP8, (7, 5, 5)), (fps.PREC_FP8, (3, 3, 3))]
    for D, a1, a2 in [(50, 0.2, 0.5), (50, 0.3, 0.7), (7, 0.34, 0.67), (3, 0.34, 0.67), (1000, 0.123, 0.9)]:
        for t in range(1, D + 1):
            prec, win = fps.schedule_select(fps.make_step_cfg(t, D, a1, a2, regimes))
            want = regimes[fo.schedule_select(t, D, a1, a2)]
            assert (prec, win) == want
    picks = [fps.schedule_select(fps.make_step_cfg(t, 50, 0.2, 0.5, regimes))[1] for t in range(1, 51)]
    assert picks == [(41, 11, 9)] * 10 + [(7, 5, 5)] * 15 + [(3, 3, 3)] * 25
    # Eq. 6 pairs each window with a tile granularity g(t): coarse, fine, intermediate
    with_g = [(fps.PREC_FP8, (3, 3, 3), (6, 8, 8)), (fps.PREC_FP8, (7, 5, 5), (1, 8, 16)),
              (fps.PREC_FP8, (5, 3, 3), (2, 8, 16))]
    tiles = [fps.schedule_select(fps.make_step_cfg(t, 50, 0.2, 0.5, with_g), with_tile=True)[2]
             for t in range(1, 51)]
    assert tiles == [(6, 8, 8)] * 10 + [(1, 8, 16)] * 15 + [(2, 8, 16)] * 25
    assert fps.schedule_select(fps.make_step_cfg(3, 50, 0.2, 0.5, regimes), with_tile=True)[2] is None
    with pytest.raises(fps.FpsError):
        fps.schedule_select(fps.make_step_cfg(3, 50, 0.2, 0.5, [(1, (3, 3, 3), (6, 0, 8))] * 3))


@pytest.mark.parametrize("bad", [dict(step=0), dict(step=51), dict(alpha1=0.6), dict(alpha2=1.0),
                                 dict(alpha1=0.0), dict(num_steps=0)])
def test_schedule_select_rejects_bad_config(bad):
    kw = dict(step=1, num_steps=50, alpha1=0.2, alpha2=0.5)
    kw.update(bad)
    cfg = fps.make_step_cfg(kw["step"], kw["num_steps"], kw["alpha1"], kw["alpha2"],
                            [(1, (3, 3, 3))] * 3)
    with pytest.raises(fps.FpsError) as e:
        fps.schedule_select(cfg)
    assert e.value.status == fps.FPS_ERR_INVALID_ARG and len(str(e.value)) > 0


@pytest.mark.parametrize("grid,tile,window", [
    ((4, 16, 16), (2, 4, 4), (1, 3, 3)),
    ((21, 30, 52), (1, 8, 16), (3, 3, 3)),
    ((21, 45, 80), (1, 8, 16), (5, 3, 3)),
    ((21, 45, 80), (1, 8, 16), (6, 6, 1)),
    ((5, 9, 33), (2, 4, 4), (2, 5, 100)),
    ((21, 30, 52), (3, 4, 4), (3, 5, 5)),          # tile shapes of the granularity ablation (Table 3)
    ((21, 30, 52), (6, 8, 8), (3, 3, 3)),
    ((21, 45, 80), (12, 16, 16), (1, 3, 3)),
    ((21, 45, 80), (24, 32, 32), (3, 3, 3)),
])
def test_tile_mask_host_matches_oracle(grid, tile, window):
    shape = fps.make_shape(2, grid, tile)
    g = fo.Geometry(*grid, *tile)
    assert fps.num_tiles(shape) == g.M
    mask, pairs = fps.tile_mask_host(shape, window)
    want = fo.tile_mask(g, window)
    assert np.array_equal(mask.astype(bool), want) and pairs == int(want.sum())
    mask_s, pairs_s = fps.tile_mask_host(shape, window + (fps.EDGE_SHIFT,))
    want_s = fo.tile_mask(g, window, edge=fo.EDGE_SHIFT)
    assert np.array_equal(mask_s.astype(bool), want_s) and pairs_s == int(want_s.sum())
    slots = fps.tile_slots(shape)                      # a tile's tokens rounded up to whole blocks
    assert slots >= g.TS and slots % 32 == 0 and slots - g.TS < 128
    assert fps.packed_bytes(shape, fps.PREC_FP8) == 2 * g.M * slots * 128
    assert fps.packed_bytes(shape, fps.PREC_BF16) == 4 * g.M * slots * 128


def test_shape_validation():
    L = fps.lib()
    ok = fps.make_shape(2, (4, 16, 16), (2, 4, 4))
    assert fps.num_tiles(ok) == 32
    assert fps.num_tiles(fps.make_shape(2, (4, 16, 16), (2, 4, 4), head_dim=64)) == 0
    assert "head_dim" in fps.last_error()
    # any tile shape up to 32768 tokens; a tile occupies whole blocks of 32 or 128 slots
    for tile, m, slots in [((1, 4, 4), 64, 32), ((2, 4, 4), 32, 32), ((3, 4, 4), 32, 64),
                           ((2, 8, 4), 16, 64), ((1, 8, 12), 16, 96), ((1, 7, 15), 24, 128),
                           ((1, 8, 16), 8, 128), ((2, 8, 12), 8, 256), ((2, 8, 16), 4, 256),
                           ((6, 8, 8), 4, 384), ((4, 16, 16), 1, 1024), ((12, 16, 16), 1, 3072),
                           ((24, 32, 32), 1, 24576), ((32, 32, 32), 1, 32768)]:
        sh = fps.make_shape(2, (4, 16, 16), tile)
        assert (fps.num_tiles(sh), fps.tile_slots(sh)) == (m, slots), tile
        assert fps.packed_bytes(sh, fps.PREC_FP8) == 2 * m * slots * 128
    # quantisation sub-tiles: each padded to whole blocks, one scale each
    for tile, qtile, groups, slots in [((2, 8, 16), (1, 8, 16), 2, 256), ((6, 8, 8), (2, 8, 8), 3, 384),
                                       ((4, 8, 8), (2, 4, 8), 4, 256), ((2, 4, 4), (1, 2, 4), 4, 128),
                                       ((2, 7, 15), (1, 7, 5), 6, 384), ((2, 8, 16), (2, 8, 16), 1, 256)]:
        sh = fps.make_shape(2, (4, 16, 16), tile, qtile=qtile)
        assert fps.num_groups(sh) == fps.num_tiles(sh) * groups and fps.tile_slots(sh) == slots, (tile, qtile)
    # the block size the library reports: 32 for groups of at most 96 tokens, else 128, and the slot
    # counts follow from it
    for tile in [(1, 4, 4), (3, 4, 4), (1, 8, 12), (1, 7, 15), (1, 8, 16), (6, 8, 8), (24, 32, 32)]:
        for qtile in [None, (1, 1, tile[2]), (1, tile[1], tile[2])]:
            sh = fps.make_shape(2, (4, 16, 16), tile, qtile=qtile)
            qs = (qtile or tile)[0] * (qtile or tile)[1] * (qtile or tile)[2]
            ns = tile[0] * tile[1] * tile[2] // qs
            bs = fps.block_slots(sh)
            assert bs == (32 if qs <= 96 else 128), (tile, qtile)
            assert fps.tile_slots(sh) == ns * -(-qs // bs) * bs, (tile, qtile)
    assert fps.num_groups(fps.make_shape(2, (4, 16, 16), (2, 8, 16))) == 4
    assert fps.num_tiles(fps.make_shape(2, (4, 16, 16), (2, 8, 16), qtile=(1, 3, 16))) == 0   # 3 does not divide 8
    assert "sub-tile" in fps.last_error()
    assert fps.num_tiles(fps.make_shape(2, (4, 16, 16), (2, 8, 16), qtile=(1, 0, 16))) == 0
    assert fps.num_tiles(fps.make_shape(2, (4, 16, 16), (33, 32, 32))) == 0   # 33792 tokens: too large
    assert "unsupported" in fps.last_error()
    assert fps.tile_slots(fps.make_shape(2, (4, 16, 16), (33, 32, 32))) == 0
    assert L.fps_block_slots(ctypes.byref(fps.make_shape(2, (4, 16, 16), (33, 32, 32)))) == 0
    assert fps.num_tiles(fps.make_shape(0, (4, 16, 16), (2, 4, 4))) == 0
    assert L.fps_num_tiles(None) == 0


def test_device_entry_points_validate_before_launching():
    """Bad arguments are refused on the host: none of these calls reaches the GPU."""
    L = fps.lib()
    shape = fps.make_shape(2, (4, 16, 16), (2, 4, 4))
    win = fps.Window(1, 3, 3)
    good = ctypes.c_void_p(0x10000)          # aligned, never dereferenced by a refused call
    odd = ctypes.c_void_p(0x10004)
    S = ctypes.byref(shape)
    assert L.fps_tile_order(S, None, good, None) == fps.FPS_ERR_INVALID_ARG
    assert "NULL" in fps.last_error()
    assert L.fps_tile_order(S, odd, good, None) == fps.FPS_ERR_INVALID_ARG
    assert "aligned" in fps.last_error()
    assert L.fps_quantize_tiles(S, good, 3, 0, good, good, None) == fps.FPS_ERR_INVALID_ARG
    assert L.fps_quantize_tiles(S, good, 2, 5, good, good, None) == fps.FPS_ERR_INVALID_ARG
    assert L.fps_quantize_tiles(S, good, 0, 0, good, None, None) == fps.FPS_ERR_INVALID_ARG
    assert L.fps_pack_tiles_bf16(S, good, -1, good, good, None) == fps.FPS_ERR_INVALID_ARG
    assert L.fps_pack_tiles_bf16(S, good, 2, good, None, None) == fps.FPS_ERR_INVALID_ARG
    assert L.fps_debug_unpack_q8(S, good, 0, odd, None) == fps.FPS_ERR_INVALID_ARG
    assert L.fps_tile_unorder(S, good, 7, good, None) == fps.FPS_ERR_INVALID_ARG
    bad_win = fps.Window(0, 3, 3)
    args = (good, good, good, good, good, good, 0, good, 1, 0, None, None)
    assert L.fps_attn_fwd(S, ctypes.byref(fps.Window(1, 3, 3, 2)), 1, None, *args) == fps.FPS_ERR_INVALID_ARG
    assert L.fps_attn_fwd(S, ctypes.byref(bad_win), 1, None, *args) == fps.FPS_ERR_INVALID_ARG
    assert L.fps_attn_fwd(S, ctypes.byref(win), 2, None, *args) == fps.FPS_ERR_INVALID_ARG
    assert L.fps_attn_fwd(S, None, 1, None, *args) == fps.FPS_ERR_INVALID_ARG
    assert L.fps_attn_fwd(S, ctypes.byref(win), 1, None, good, good, good, None, good, good, 0,
                          good, 1, 0, None, None) == fps.FPS_ERR_INVALID_ARG   # FP8 needs scales
    assert L.fps_attn_fwd(S, ctypes.byref(win), 1, None, good, good, good, good, good, good, 0,
                          good, 1, 2, None, None) == fps.FPS_ERR_INVALID_ARG   # bad output layout
    assert L.fps_quantize_raster(S, good, 0, 0, None, good, None) == fps.FPS_ERR_INVALID_ARG
    assert L.fps_debug_mfma_rate(0, 4, good, None) == fps.FPS_ERR_INVALID_ARG
    assert L.fps_debug_mfma_rate(4, 0, good, None) == fps.FPS_ERR_INVALID_ARG
    assert L.fps_debug_mfma_rate(4, 4, None, None) == fps.FPS_ERR_INVALID_ARG
    assert L.fps_debug_issue_mix(5, 0, 0, 1, 4, 4, good, good, None) == fps.FPS_ERR_INVALID_ARG
    assert L.fps_debug_issue_mix(0, 0, 2, 1, 4, 4, good, good, None) == fps.FPS_ERR_INVALID_ARG
    assert L.fps_debug_issue_mix(0, 0, 0, 9, 4, 4, good, good, None) == fps.FPS_ERR_INVALID_ARG
    assert L.fps_debug_issue_mix(0, 0, 0, 1, 4, 4, None, good, None) == fps.FPS_ERR_INVALID_ARG
    assert L.fps_debug_copy(good, good, 24, None) == fps.FPS_ERR_INVALID_ARG
    assert L.fps_debug_copy(good, None, 32, None) == fps.FPS_ERR_INVALID_ARG
    big = fps.make_shape(2, (64, 64, 64), (64, 32, 32))                         # 65536-token tiles
    assert L.fps_attn_fwd(ctypes.byref(big), ctypes.byref(win), 1, None, *args) == fps.FPS_ERR_UNSUPPORTED
    big = fps.make_shape(2, (24, 32, 32), (24, 32, 32))        # score debug call: at most 4096 slots
    assert L.fps_debug_scores_q8(ctypes.byref(big), good, good, 0, 0, 0, good, None) == fps.FPS_ERR_UNSUPPORTED
    cfg = fps.make_step_cfg(99, 50, 0.2, 0.5, [(1, (3, 3, 3))] * 3)
    assert L.fps_attn_fwd(S, None, 1, ctypes.byref(cfg), *args) == fps.FPS_ERR_INVALID_ARG
    # a regime that names a tile must be called with inputs of that tile
    cfg = fps.make_step_cfg(5, 50, 0.2, 0.5, [(1, (3, 3, 3), (shape.Tt + 1, shape.Th, shape.Tw))] * 3)
    assert L.fps_attn_fwd(S, None, 1, ctypes.byref(cfg), *args) == fps.FPS_ERR_INVALID_ARG
    assert "selects tile" in fps.last_error()


def test_reciprocal_division_identity_used_by_the_kernels():
    """The kernels decode slot ranks with q = int((n + 0.5f) * (1.0f / d)) in float32 instead of an
    integer division.  The identity q == n // d is checked here at every multiple of d and its
    neighbours (where a rounding error would show first) for all divisors a tile can have."""
    for d in list(range(1, 2049)) + list(range(2049, 32769, 97)) + [32768]:
        inv = np.float32(1.0) / np.float32(d)
        k = np.arange(0, (1 << 17) // d + 2, dtype=np.int64)
        n = np.unique(np.clip(np.concatenate([k * d - 1, k * d, k * d + 1, k * d + d // 2]), 0, (1 << 17) - 1))
        q = ((n.astype(np.float32) + np.float32(0.5)) * inv).astype(np.int64)
        assert np.array_equal(q, n // d), d
