"""Thin ctypes binding over libfps (argument marshalling only; every step runs in the HIP kernels).

PyTorch is used for device memory and streams.  There is no CPU fallback: if the shared library
has not been built (see `paper_2506_04648_amd.build`), loading fails with an error.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfps.so")

FPS_OK = 0
FPS_ERR_INVALID_ARG = -1
FPS_ERR_UNSUPPORTED = -2
FPS_ERR_WORKSPACE = -3
FPS_ERR_HIP = -4

PREC_BF16, PREC_FP8 = 0, 1
VSCALE_TILE, VSCALE_CHANNEL = 0, 1
ROLE_Q, ROLE_K, ROLE_V = 0, 1, 2
OUT_BF16, OUT_F32 = 0, 1
LAYOUT_TILED, LAYOUT_RASTER = 0, 1
EDGE_TRUNCATE, EDGE_SHIFT = 0, 1

EXPORTS = ("fps_last_error", "fps_schedule_select", "fps_num_tiles", "fps_num_groups", "fps_tile_slots",
           "fps_block_slots", "fps_packed_bytes",
           "fps_tile_mask_host", "fps_tile_order", "fps_tile_unorder", "fps_quantize_tiles",
           "fps_quantize_raster",
           "fps_pack_tiles_bf16", "fps_pack_raster_bf16", "fps_debug_unpack_q8", "fps_debug_copy", "fps_debug_scores_q8",
           "fps_debug_scores_block_q8", "fps_debug_mfma_rate", "fps_debug_issue_mix",
           "fps_attn_fwd")


class Shape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in ("B", "heads", "head_dim", "T", "H", "W", "Tt", "Th", "Tw",
                                            "Qt", "Qh", "Qw")]


class Window(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in ("wt", "wh", "ww", "edge")]


class Regime(ctypes.Structure):
    _fields_ = [("prec", ctypes.c_int), ("win", Window)] + [(n, ctypes.c_int) for n in
                                                            ("Tt", "Th", "Tw", "Qt", "Qh", "Qw")]


class StepCfg(ctypes.Structure):
    _fields_ = [("step", ctypes.c_int), ("num_steps", ctypes.c_int), ("alpha1", ctypes.c_float),
                ("alpha2", ctypes.c_float), ("regime", Regime * 3)]


class FpsError(RuntimeError):
    def __init__(self, status, text):
        super().__init__(f"libfps status {status}: {text}")
        self.status = status


_lib = None


def lib():
    """Load libfps.so (once).  Raises if it is not built: the product path has no fallback."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} not found: build it with `python -c 'import __graft_entry__ as g; g.build()'`")
        L = ctypes.CDLL(LIB_PATH)
        vp, ip, fp = ctypes.c_void_p, ctypes.c_int, ctypes.POINTER(ctypes.c_float)
        L.fps_last_error.restype = ctypes.c_char_p
        L.fps_last_error.argtypes = []
        L.fps_schedule_select.argtypes = [ctypes.POINTER(StepCfg), ctypes.POINTER(Regime)]
        L.fps_num_tiles.restype = ctypes.c_size_t
        L.fps_num_tiles.argtypes = [ctypes.POINTER(Shape)]
        L.fps_num_groups.restype = ctypes.c_size_t
        L.fps_num_groups.argtypes = [ctypes.POINTER(Shape)]
        L.fps_tile_slots.restype = ctypes.c_size_t
        L.fps_tile_slots.argtypes = [ctypes.POINTER(Shape)]
        L.fps_block_slots.restype = ctypes.c_size_t
        L.fps_block_slots.argtypes = [ctypes.POINTER(Shape)]
        L.fps_packed_bytes.restype = ctypes.c_size_t
        L.fps_packed_bytes.argtypes = [ctypes.POINTER(Shape), ip]
        L.fps_tile_mask_host.argtypes = [ctypes.POINTER(Shape), ctypes.POINTER(Window), vp,
                                         ctypes.POINTER(ctypes.c_uint64)]
        L.fps_tile_order.argtypes = [ctypes.POINTER(Shape), vp, vp, vp]
        L.fps_tile_unorder.argtypes = [ctypes.POINTER(Shape), vp, ip, vp, vp]
        L.fps_quantize_tiles.argtypes = [ctypes.POINTER(Shape), vp, ip, ip, vp, vp, vp]
        L.fps_quantize_raster.argtypes = [ctypes.POINTER(Shape), vp, ip, ip, vp, vp, vp]
        L.fps_pack_tiles_bf16.argtypes = [ctypes.POINTER(Shape), vp, ip, vp, vp, vp]
        L.fps_pack_raster_bf16.argtypes = [ctypes.POINTER(Shape), vp, ip, vp, vp, vp]
        L.fps_debug_unpack_q8.argtypes = [ctypes.POINTER(Shape), vp, ip, vp, vp]
        L.fps_debug_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
        L.fps_debug_scores_q8.argtypes = [ctypes.POINTER(Shape), vp, vp, ip, ip, ip, vp, vp]
        L.fps_debug_scores_block_q8.argtypes = [ctypes.POINTER(Shape), vp, vp, ip, ip, ip, ip, ip, vp,
                                                ctypes.POINTER(ctypes.c_int), vp]
        L.fps_debug_mfma_rate.argtypes = [ip, ip, vp, vp]
        L.fps_debug_issue_mix.argtypes = [ip, ip, ip, ip, ip, ip, vp, vp, vp]
        L.fps_attn_fwd.argtypes = [ctypes.POINTER(Shape), ctypes.POINTER(Window), ip,
                                   ctypes.POINTER(StepCfg), vp, vp, vp, vp, vp, vp, ip, vp, ip, ip, vp, vp]
        for name in EXPORTS:
            if name not in ("fps_last_error", "fps_num_tiles", "fps_num_groups", "fps_tile_slots",
                            "fps_block_slots", "fps_packed_bytes"):
                getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def last_error() -> str:
    return lib().fps_last_error().decode()


def _check(status):
    if status != FPS_OK:
        raise FpsError(status, last_error())


def make_shape(heads, grid, tile, B=1, head_dim=128, qtile=None) -> Shape:
    """qtile: quantisation sub-tile (it must divide the tile); None = one scale per tile."""
    q = (0, 0, 0) if qtile is None else tuple(qtile)
    return Shape(B, heads, head_dim, grid[0], grid[1], grid[2], tile[0], tile[1], tile[2], q[0], q[1], q[2])


def make_step_cfg(step, num_steps, alpha1, alpha2, regimes) -> StepCfg:
    """regimes: three (prec, (wt, wh, ww[, edge])[, (Tt, Th, Tw)[, (Qt, Qh, Qw)]]) entries for the
    early, mid and late steps (Eq. 6); the optional items are the regime's granularity g(t): its
    tile and its quantisation sub-tile."""
    cfg = StepCfg()
    cfg.step, cfg.num_steps, cfg.alpha1, cfg.alpha2 = step, num_steps, alpha1, alpha2
    for i, reg in enumerate(regimes):
        cfg.regime[i].prec = reg[0]
        cfg.regime[i].win = Window(*reg[1])
        if len(reg) > 2 and reg[2] is not None:
            cfg.regime[i].Tt, cfg.regime[i].Th, cfg.regime[i].Tw = reg[2]
        if len(reg) > 3 and reg[3] is not None:
            cfg.regime[i].Qt, cfg.regime[i].Qh, cfg.regime[i].Qw = reg[3]
    return cfg


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else None


# ---- host helpers ---------------------------------------------------------------------------
def schedule_select(cfg: StepCfg, with_tile=False):
    """(prec, window) of the step's regime; with_tile=True appends its tile (Tt, Th, Tw) or None,
    and its quantisation sub-tile if it names one."""
    out = Regime()
    _check(lib().fps_schedule_select(ctypes.byref(cfg), ctypes.byref(out)))
    win = (out.win.wt, out.win.wh, out.win.ww) + ((out.win.edge,) if out.win.edge else ())
    if with_tile:
        tile = (out.Tt, out.Th, out.Tw) if out.Tt else None
        if out.Qt:
            return out.prec, win, tile, (out.Qt, out.Qh, out.Qw)
        return out.prec, win, tile
    return out.prec, win


def num_tiles(shape: Shape) -> int:
    return int(lib().fps_num_tiles(ctypes.byref(shape)))


def num_groups(shape: Shape) -> int:
    """Quantisation groups (scales) per head: one per tile, or per sub-tile of each tile."""
    return int(lib().fps_num_groups(ctypes.byref(shape)))


def tile_slots(shape: Shape) -> int:
    """Slots one tile occupies in tiled and packed tensors (its tokens rounded up to whole blocks)."""
    return int(lib().fps_tile_slots(ctypes.byref(shape)))


def packed_bytes(shape: Shape, prec: int) -> int:
    return int(lib().fps_packed_bytes(ctypes.byref(shape), prec))


def tile_mask_host(shape: Shape, window):
    import numpy as np
    M = num_tiles(shape)
    if M == 0:
        raise FpsError(FPS_ERR_INVALID_ARG, last_error())
    mask = np.zeros((M, M), dtype=np.uint8)
    pairs = ctypes.c_uint64(0)
    win = Window(*window)
    _check(lib().fps_tile_mask_host(ctypes.byref(shape), ctypes.byref(win),
                                    mask.ctypes.data_as(ctypes.c_void_p), ctypes.byref(pairs)))
    return mask, int(pairs.value)


# ---- device entry points (torch tensors on the current device) --------------------------------
def _tiled_len(shape: Shape) -> int:
    n = num_tiles(shape) * tile_slots(shape)
    if n == 0:
        raise FpsError(FPS_ERR_INVALID_ARG, last_error())
    return n


def tile_order(shape: Shape, x_raster, out=None):
    import torch
    assert x_raster.dtype == torch.bfloat16 and x_raster.is_cuda and x_raster.is_contiguous()
    if out is None:
        out = torch.empty((shape.B, shape.heads, _tiled_len(shape), shape.head_dim),
                          dtype=torch.bfloat16, device=x_raster.device)
    _check(lib().fps_tile_order(ctypes.byref(shape), _ptr(x_raster), _ptr(out), _stream()))
    return out


def tile_unorder(shape: Shape, o_tiled, out=None):
    import torch
    assert o_tiled.is_cuda and o_tiled.is_contiguous()
    dt = OUT_F32 if o_tiled.dtype == torch.float32 else OUT_BF16
    if out is None:
        out = torch.empty((shape.B, shape.heads, shape.T, shape.H, shape.W, shape.head_dim),
                          dtype=o_tiled.dtype, device=o_tiled.device)
    _check(lib().fps_tile_unorder(ctypes.byref(shape), _ptr(o_tiled), dt, _ptr(out), _stream()))
    return out


def quantize_tiles(shape: Shape, x_tiled, role, vscale=VSCALE_TILE, out=None, scales=None,
                   raster=False):
    """Per-tile FP8 quantisation of a tile-ordered tensor, or (raster=True) of a raster tensor with
    the tile ordering fused in.  Returns (packed codes, scales)."""
    import torch
    assert x_tiled.dtype == torch.bfloat16 and x_tiled.is_cuda and x_tiled.is_contiguous()
    if out is None:
        out = torch.empty(packed_bytes(shape, PREC_FP8), dtype=torch.uint8, device=x_tiled.device)
    if scales is None:
        n = shape.head_dim if (role == ROLE_V and vscale == VSCALE_CHANNEL) else num_groups(shape)
        scales = torch.empty((shape.B, shape.heads, n), dtype=torch.float32, device=x_tiled.device)
    fn = lib().fps_quantize_raster if raster else lib().fps_quantize_tiles
    _check(fn(ctypes.byref(shape), _ptr(x_tiled), role, vscale, _ptr(out), _ptr(scales), _stream()))
    return out, scales


def pack_tiles_bf16(shape: Shape, x_tiled, role, out=None, vscale=None, raster=False):
    """BF16-mode operand packing of a tile-ordered tensor, or (raster=True) of a raster tensor with
    the tile ordering fused in.  Returns (packed tensor, per-group V scales or None)."""
    import torch
    assert x_tiled.dtype == torch.bfloat16 and x_tiled.is_cuda and x_tiled.is_contiguous()
    if out is None:
        out = torch.empty(packed_bytes(shape, PREC_BF16), dtype=torch.uint8, device=x_tiled.device)
    if role == ROLE_V and vscale is None:
        vscale = torch.empty((shape.B, shape.heads, num_groups(shape)), dtype=torch.float32,
                             device=x_tiled.device)
    fn = lib().fps_pack_raster_bf16 if raster else lib().fps_pack_tiles_bf16
    _check(fn(ctypes.byref(shape), _ptr(x_tiled), role, _ptr(out), _ptr(vscale), _stream()))
    return out, vscale


def debug_unpack_q8(shape: Shape, xq, role):
    import torch
    out = torch.empty((shape.B, shape.heads, _tiled_len(shape), shape.head_dim), dtype=torch.uint8,
                      device=xq.device)
    _check(lib().fps_debug_unpack_q8(ctypes.byref(shape), _ptr(xq), role, _ptr(out), _stream()))
    return out


def debug_copy(src, dst):
    assert src.is_cuda and dst.is_cuda and src.is_contiguous() and dst.is_contiguous()
    nbytes = src.numel() * src.element_size()
    assert nbytes == dst.numel() * dst.element_size()
    _check(lib().fps_debug_copy(_ptr(src), _ptr(dst), nbytes, _stream()))
    return dst


def debug_mfma_rate(workgroups, iters, sink):
    """Launch the MFMA-only kernel; returns the FLOPs it executes (the caller times it)."""
    assert sink.is_cuda and sink.numel() >= workgroups * 256
    _check(lib().fps_debug_mfma_rate(workgroups, iters, _ptr(sink), _stream()))
    return workgroups * 4 * iters * 8 * 65536.0


def debug_issue_mix(matrix_kind, valu_per_mfma, valu_kind, workgroups_per_cu, workgroups, iters, sink, cycles):
    """One launch of the matrix/vector issue-mix kernel; cycles (int64, workgroups*4) receives each
    wave's shader clocks for iters*8 groups."""
    _check(lib().fps_debug_issue_mix(matrix_kind, valu_per_mfma, valu_kind, workgroups_per_cu, workgroups,
                                     iters, _ptr(sink), _ptr(cycles), _stream()))


def debug_scores_q8(shape: Shape, q8, k8, bh, u, v):
    import torch
    ts = tile_slots(shape)
    out = torch.empty((ts, ts), dtype=torch.float32, device=q8.device)
    _check(lib().fps_debug_scores_q8(ctypes.byref(shape), _ptr(q8), _ptr(k8), bh, u, v, _ptr(out),
                                     _stream()))
    return out


def block_slots(shape: Shape) -> int:
    """BS, the slots of one block, as the library lays tensors out (128 or 32)."""
    n = lib().fps_block_slots(ctypes.byref(shape))
    if n == 0:
        raise FpsError(FPS_ERR_INVALID_ARG, last_error())
    return int(n)


def debug_scores_block_q8(shape: Shape, q8, k8, bh, u, jq, v, jk, out=None):
    """Raw score accumulators of one (query block, key block) pair; returns a [BS, BS] tensor."""
    import torch
    bs = block_slots(shape)
    if out is None:
        out = torch.empty((bs, bs), dtype=torch.float32, device=q8.device)
    got = ctypes.c_int(0)
    _check(lib().fps_debug_scores_block_q8(ctypes.byref(shape), _ptr(q8), _ptr(k8), bh, u, jq, v, jk,
                                           _ptr(out), ctypes.byref(got), _stream()))
    assert got.value == bs
    return out


def attn_fwd(shape: Shape, window, prec, q, k, v, sq=None, sk=None, sv=None, vscale=VSCALE_TILE,
             out=None, out_dtype=None, visited=None, step: StepCfg = None, raster_out=False):
    import torch
    if out is None:
        out_dtype = out_dtype or torch.bfloat16
        dims = ((shape.T, shape.H, shape.W, shape.head_dim) if raster_out
                else (_tiled_len(shape), shape.head_dim))
        out = torch.empty((shape.B, shape.heads) + dims, dtype=out_dtype, device=q.device)
    dt = OUT_F32 if out.dtype == torch.float32 else OUT_BF16
    win = Window(*window) if window is not None else None
    if win is None and step is None:
        raise ValueError("attn_fwd needs a window or a step configuration")
    _check(lib().fps_attn_fwd(ctypes.byref(shape), ctypes.byref(win) if win is not None else None,
                              prec, ctypes.byref(step) if step is not None else None,
                              _ptr(q), _ptr(k), _ptr(v), _ptr(sq), _ptr(sk), _ptr(sv), vscale,
                              _ptr(out), dt, LAYOUT_RASTER if raster_out else LAYOUT_TILED,
                              _ptr(visited), _stream()))
    return out
