"""Seeded synthetic Q/K/V generator shared by the tests, the benchmark and the smoke check.

This module holds none of the method's arithmetic: it only draws random numbers, scales a few
"outlier" channels and rounds to bf16-representable float32.  Both the CPU oracle and the HIP
path are fed from here so that they see bit-identical inputs.  It imports nothing from the rest
of the package and nothing from the oracle.

Recipe (stands in for Wan2.1 activations; shapes follow the paper's hyper-parameter appendix:
12 or 40 heads, head_dim 128, up to 75600 tokens):
  * one independent PCG64 stream per (config, call, tensor, head), seeded from
    SeedSequence([BASE_SEED, config_id, call_index, tensor_id, head]);
  * float32 standard normal over the real (un-padded) raster grid [T, H, W, d];
  * `n_outlier` channels per (tensor, head), chosen without replacement from that stream after
    the normal draw, are multiplied by 8;
  * round-to-nearest-even to bf16, returned as float32 holding the bf16 value exactly.
"""
from __future__ import annotations

import dataclasses
import numpy as np

BASE_SEED = 20250604
HEAD_DIM = 128


@dataclasses.dataclass(frozen=True)
class Workload:
    """One benchmark / parity configuration (token grid, tile, window, heads)."""
    name: str
    config_id: int
    heads: int
    grid: tuple          # (T, H, W) real token grid
    tile: tuple          # (Tt, Th, Tw)
    window: tuple        # (wt, wh, ww) in tiles
    n_outlier: int
    head_dim: int = HEAD_DIM
    batch: int = 1


TINY = Workload("tiny", 1, 2, (4, 16, 16), (2, 4, 4), (1, 3, 3), 4)
WAN_1_3B_480P = Workload("wan1.3b-480p", 2, 12, (21, 30, 52), (1, 8, 16), (3, 3, 3), 3)
WAN_14B_720P = Workload("wan14b-720p", 3, 40, (21, 45, 80), (1, 8, 16), (5, 3, 3), 3)
WAN_14B_720P_DENSE = dataclasses.replace(WAN_14B_720P, name="wan14b-720p-dense", config_id=4,
                                         window=(41, 11, 9))
WAN_14B_720P_MID = dataclasses.replace(WAN_14B_720P, name="wan14b-720p-win755", config_id=5,
                                       window=(7, 5, 5))
WAN_14B_720P_LATE = dataclasses.replace(WAN_14B_720P, name="wan14b-720p-win333", config_id=5,
                                        window=(3, 3, 3))

WORKLOADS = {w.name: w for w in (TINY, WAN_1_3B_480P, WAN_14B_720P, WAN_14B_720P_DENSE,
                                 WAN_14B_720P_MID, WAN_14B_720P_LATE)}


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """float32 -> nearest bf16 (ties to even), returned as float32 (finite inputs only)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    u = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return u.view(np.float32)


def head_tensor(config_id: int, call_index: int, tensor_id: int, head: int, grid, head_dim: int,
                n_outlier: int, outlier_gain: float = 8.0) -> np.ndarray:
    """One head of one tensor (tensor_id 0/1/2 = Q/K/V) in raster order: float32 [T, H, W, d]."""
    ss = np.random.SeedSequence([BASE_SEED, config_id, call_index, tensor_id, head])
    rng = np.random.Generator(np.random.PCG64(ss))
    T, H, W = grid
    x = rng.standard_normal((T, H, W, head_dim), dtype=np.float32)
    if n_outlier > 0:
        ch = rng.choice(head_dim, size=n_outlier, replace=False)
        x[..., ch] *= np.float32(outlier_gain)
    return round_to_bf16(x)


def qkv_raster(w: Workload, call_index: int = 0, heads=None, workers: int = 1):
    """Q, K, V as float32 arrays [n_heads_selected, T, H, W, d] holding bf16 values (B = 1).
    `workers` > 1 draws the independent (tensor, head) streams on a thread pool; the result does
    not depend on it."""
    heads = list(range(w.heads) if heads is None else heads)
    jobs = [(tensor_id, h) for tensor_id in range(3) for h in heads]

    def one(job):
        return head_tensor(w.config_id, call_index, job[0], job[1], w.grid, w.head_dim, w.n_outlier)

    if workers > 1:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=workers) as pool:
            parts = list(pool.map(one, jobs))
    else:
        parts = [one(j) for j in jobs]
    n = len(heads)
    return tuple(np.stack(parts[t * n:(t + 1) * n]) for t in range(3))
