#!/usr/bin/env python3
"""Benchmark of the FP8 3D sliding-tile attention hot path on one MI355X.

One "step" is one pass of the whole path over one batch of synthetic Wan2.1-14B 720p-shaped inputs
already resident in HBM in raster order: tile ordering + per-tile FP8 quantisation of Q, K, V (one
fused kernel per tensor) and the sliding-tile attention kernel, whose epilogue writes the output
back in raster order.  Prints ONE JSON line.

After the timed steps the same process also times, each outside the headline figure: the dense BF16
and dense FP8 launches on the same grid (the speed-up's reference points), the 50-call
denoising-step-aware schedule (Eq. 6) on fresh inputs per call, and the CPU oracle on a bounded
sample.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-dense] [--no-cpu]
                  [--no-schedule] [--variants] [--window-ablation]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

FP8_PEAK_TFLOPS = 5000.0     # MI355X dense FP8 MFMA, published
BF16_PEAK_TFLOPS = 2500.0
HBM_PEAK_GBPS = 8000.0       # MI355X HBM3E, published
# HBM bytes per launch of the attention kernel: rocprofv3 FETCH_SIZE and WRITE_SIZE, each scaled by
# what the same counter reads for a plain 1 GiB copy kernel.  Taken from the committed profile, NOT
# measured by this run (a counter run cannot share a process with the timing); the launches of one
# profile run spread as stated there.
PROFILED_TRAFFIC = {"wan14b-720p": {"bytes": 2.36e9, "range": [2.358e9, 2.362e9],
                                    "source": "profiles/attn_fp8_wan14b-720p_counters.md"}}


def kept_pairs(grid, tile, window):
    n = [-(-g // t) for g, t in zip(grid, tile)]
    total = 1
    for na, w in zip(n, window):
        r = min(w // 2, na - 1)
        total *= na * (2 * r + 1) - r * (r + 1)
    return total, n[0] * n[1] * n[2]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="wan14b-720p")
    ap.add_argument("--no-dense", action="store_true", help="skip the dense BF16 / dense FP8 reference runs")
    ap.add_argument("--no-cpu", action="store_true", help="skip the timed CPU oracle sample")
    ap.add_argument("--cpu-heads", type=int, default=4, help="heads in the timed CPU oracle sample")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also launch one plain 1 GiB device copy (reference for the profiler's traffic counters)")
    ap.add_argument("--no-schedule", action="store_true",
                    help="skip the 50-call denoising-step-aware schedule (Eq. 6), e.g. under a profiler")
    ap.add_argument("--schedule", action="store_true", help="(the schedule runs by default; kept for old command lines)")
    ap.add_argument("--variants", action="store_true",
                    help="also time the variants of the path on the same grid: per-channel V scales, BF16 with "
                         "the sparse window, the shifted-window edge rule, other tile shapes")
    ap.add_argument("--window-ablation", action="store_true",
                    help="also time the window sizes of the paper's window ablation (Table 4) on the "
                         "Wan2.1-1.3B 480p grid, against the dense BF16 kernel on the same grid")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (heads are independent and would shard across "
              "GPUs without any exchange); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2506_04648_amd import fps, synth

    fps.lib()                                            # no fallback: fail now if not built
    w = synth.WORKLOADS[args.workload]
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    shape = fps.make_shape(w.heads, w.grid, w.tile)
    pairs, M = kept_pairs(w.grid, w.tile, w.window)
    TS = w.tile[0] * w.tile[1] * w.tile[2]
    flop = pairs * w.heads * 4.0 * TS * TS * w.head_dim          # QK^T and PV on computed tiles

    t0 = time.time()
    q, k, v = synth.qkv_raster(w, workers=min(16, os.cpu_count() or 1))
    raster = [torch.from_numpy(a[None]).to(dev).to(torch.bfloat16) for a in (q, k, v)]
    del q, k, v
    gen_s = time.time() - t0

    # persistent buffers: the timed region allocates nothing
    L = M * fps.tile_slots(shape)
    packed = [torch.empty(fps.packed_bytes(shape, fps.PREC_FP8), dtype=torch.uint8, device=dev) for _ in range(3)]
    scales = [torch.empty((1, w.heads, M), dtype=torch.float32, device=dev) for _ in range(3)]
    out_raster = torch.empty((1, w.heads) + tuple(w.grid) + (128,), dtype=torch.bfloat16, device=dev)
    ev = lambda: torch.cuda.Event(enable_timing=True)

    def step(events=None):
        if events:
            events[0].record()
        for i in range(3):
            fps.quantize_tiles(shape, raster[i], i, out=packed[i], scales=scales[i], raster=True)
        if events:
            events[1].record()
        fps.attn_fwd(shape, w.window, fps.PREC_FP8, packed[0], packed[1], packed[2],
                     scales[0], scales[1], scales[2], out=out_raster, raster_out=True)
        if events:
            events[2].record()

    if args.copy_calibration:
        a_ = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(3)
        b_ = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        fps.debug_copy(a_, b_)
        torch.cuda.synchronize()
        del a_, b_
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    all_events = [[ev() for _ in range(3)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(all_events[i])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps
    seg = np.array([[e[j].elapsed_time(e[j + 1]) for j in range(2)] for e in all_events])
    quant_ms, attn_ms = (float(x) for x in seg.mean(axis=0))
    quant_med, attn_med = (float(x) for x in np.median(seg, axis=0))

    # FLOPs on real tokens only: 4 d * (real query tokens of u) * (real key tokens of v) per kept pair
    mask, _ = fps.tile_mask_host(shape, w.window)
    per_axis = [np.minimum(t, g - np.arange(-(-g // t)) * t) for g, t in zip(w.grid, w.tile)]
    real = (per_axis[0][:, None, None] * per_axis[1][None, :, None] * per_axis[2][None, None, :]).reshape(-1)
    useful_flop = 4.0 * w.head_dim * w.heads * float(real.astype(np.float64) @ mask.astype(np.float64) @ real.astype(np.float64))

    # the matrix rate the chip sustains on the attention kernel's own instruction (nothing else running)
    sink = torch.empty(4096 * 256, dtype=torch.float32, device=dev)
    fps.debug_mfma_rate(4096, 2000, sink)
    torch.cuda.synchronize()
    m0, m1 = ev(), ev()
    m0.record()
    mfma_flop = fps.debug_mfma_rate(4096, 2000, sink)
    m1.record()
    torch.cuda.synchronize()
    mfma_sustained = mfma_flop / (m0.elapsed_time(m1) * 1e-3) / 1e12
    del sink

    # The same launch on all-zero operands: identical instruction stream, work items and memory
    # traffic, but no switching activity in the matrix and vector data paths.  What it gains over the
    # real data is the shader clock the chip's power management takes away under load.
    zero_codes = torch.zeros_like(packed[0])
    one_scales = torch.ones_like(scales[0])

    def attn_zero():
        fps.attn_fwd(shape, w.window, fps.PREC_FP8, zero_codes, zero_codes, zero_codes,
                     one_scales, one_scales, one_scales, out=out_raster, raster_out=True)
    for _ in range(3):
        attn_zero()
    z0, z1 = ev(), ev()
    z0.record()
    for _ in range(10):
        attn_zero()
    z1.record()
    torch.cuda.synchronize()
    attn_zero_ms = z0.elapsed_time(z1) / 10
    del zero_codes, one_scales

    # bytes the three quantise launches really move: the un-padded bf16 raster read, the packed codes
    # (padded to whole tiles) and the scales written
    tokens = w.grid[0] * w.grid[1] * w.grid[2]
    quant_bytes = 3.0 * w.heads * (2.0 * tokens * 128 + 1.0 * L * 128 + 4.0 * M)
    traffic = PROFILED_TRAFFIC.get(w.name, {})

    result = {
        "metric": "effective TFLOP/s + ms/call, FP8 3D sliding-tile attention, Wan-14B 720p shape",
        "value": flop / (ms_per_step * 1e-3) / 1e12,
        "unit": "TFLOP/s (computed tile pairs; whole hot path: fused tile-order+quantise x3, attention)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "fp8_e4m3 (fp32 accumulate)", "data": "synthetic",
        "config": {"workload": w.name, "heads": w.heads, "head_dim": w.head_dim, "grid": list(w.grid),
                   "tile": list(w.tile), "window_tiles": list(w.window), "kept_tile_pairs": pairs,
                   "tflop_per_call": flop / 1e12, "input_gen_s": round(gen_s, 1)},
        "breakdown_ms": {"tile_order_quantize_x3": quant_ms, "attention_raster_out": attn_ms},
        "breakdown_median_ms": {"tile_order_quantize_x3": quant_med, "attention_raster_out": attn_med},
        "attention_tflops": flop / (attn_ms * 1e-3) / 1e12,
        "attention_tflops_real_tokens_only": useful_flop / (attn_ms * 1e-3) / 1e12,
        "attention_ms_all_zero_operands": attn_zero_ms,
        "mfma_only_sustained_tflops": mfma_sustained,
        "attention_frac_of_sustained_mfma": flop / (attn_ms * 1e-3) / 1e12 / mfma_sustained,
        "quantize_GBps": quant_bytes / (quant_ms * 1e-3) / 1e9,
        "roofline": {"bound": "mfma", "kernel": "attn_fp8_wide_kernel", "achieved": flop / (attn_ms * 1e-3) / 1e12,
                     "peak": FP8_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": flop / (attn_ms * 1e-3) / 1e12 / FP8_PEAK_TFLOPS,
                     "traffic": traffic.get("bytes"), "traffic_range": traffic.get("range"),
                     "traffic_source": traffic.get("source", "not profiled for this workload"),
                     "algorithmic_bytes": 3.0 * w.heads * L * 128 + 2.0 * w.heads * tokens * 128},
        # second entry: the quantise pass is the HBM-bound kernel of the path (three launches per step)
        "roofline_quantize": {"bound": "hbm", "kernel": "quantize_tiles_kernel (x3: Q, K, V)",
                              "achieved": quant_bytes / (quant_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBPS,
                              "unit": "GB/s", "frac": quant_bytes / (quant_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                              "traffic": None, "algorithmic_bytes": quant_bytes},
        "paper_context": {"kernel_speedup_vs_bf16_H20": 7.09, "e2e_speedup_vs_bf16_H20": 4.96},
    }

    if not args.no_dense:
        dense_win = tuple(2 * (-(-g // t)) - 1 for g, t in zip(w.grid, w.tile))
        dpairs, _ = kept_pairs(w.grid, w.tile, dense_win)
        dflop = dpairs * w.heads * 4.0 * TS * TS * w.head_dim

        def timed(fn, reps):
            fn()
            torch.cuda.synchronize()
            a, b = ev(), ev()
            a.record()
            for _ in range(reps):
                fn()
            b.record()
            torch.cuda.synchronize()
            return a.elapsed_time(b) / reps

        out_tiled = torch.empty((1, w.heads, L, 128), dtype=torch.bfloat16, device=dev)
        p16 = [fps.pack_tiles_bf16(shape, raster[i], i, raster=True) for i in range(3)]
        bf16_ms = timed(lambda: fps.attn_fwd(shape, dense_win, fps.PREC_BF16, p16[0][0], p16[1][0], p16[2][0],
                                             sv=p16[2][1], out=out_tiled), 2)
        # the same launch on all-zero operands (see attention_ms_all_zero_operands)
        z16 = torch.zeros_like(p16[0][0])
        one_sv = torch.ones_like(p16[2][1])
        bf16_zero_ms = timed(lambda: fps.attn_fwd(shape, dense_win, fps.PREC_BF16, z16, z16, z16, sv=one_sv,
                                                  out=out_tiled), 2)
        del p16, z16, one_sv
        fp8d_ms = timed(lambda: fps.attn_fwd(shape, dense_win, fps.PREC_FP8, packed[0], packed[1], packed[2],
                                             scales[0], scales[1], scales[2], out=out_tiled), 2)
        result["dense"] = {"window_tiles": list(dense_win), "tflop_per_call": dflop / 1e12,
                           "bf16_ms": bf16_ms, "bf16_tflops": dflop / bf16_ms / 1e9,
                           "bf16_frac_of_peak": dflop / bf16_ms / 1e9 / BF16_PEAK_TFLOPS,
                           "bf16_ms_all_zero_operands": bf16_zero_ms,
                           "fp8_ms": fp8d_ms, "fp8_tflops": dflop / fp8d_ms / 1e9}
        result["speedup_vs_own_dense_bf16"] = {"attention_only": bf16_ms / attn_ms,
                                               "with_quantize": bf16_ms / (attn_ms + quant_ms)}

    if args.variants:
        result["variants"] = run_variants(w, raster, dev)

    if args.window_ablation:
        result["window_ablation"] = run_window_ablation(dev)

    if not args.no_schedule:
        del raster, packed, scales, out_raster
        torch.cuda.empty_cache()
        result["schedule"] = run_schedule(w, shape, dev)

    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(w, args.cpu_heads, TS)

    print(json.dumps(result))


def run_variants(w, raster, dev, reps=5):
    """Variants of the hot path on the workload's grid and inputs, each timed as a whole (operand
    preparation from the raster tensors + attention with raster output): the paper's per-channel V
    scales, BF16 operands with the same sparse window, the shifted-window edge rule, and other tile
    shapes (the tile is the quantisation group and the sparsity unit; windows chosen to cover about
    the same token neighbourhood as the workload's own).  TFLOP/s counts 4*TS^2*d per kept tile pair
    with TS the tile's TOKENS (padding slots of a tile that is not a whole number of blocks are
    executed but not counted)."""
    import torch
    from paper_2506_04648_amd import fps
    out = torch.empty((1, w.heads) + tuple(w.grid) + (128,), dtype=torch.bfloat16, device=dev)
    ev = lambda: torch.cuda.Event(enable_timing=True)

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        a, b = ev(), ev()
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    def fp8_case(name, tile, window, vscale=fps.VSCALE_TILE):
        shape = fps.make_shape(w.heads, w.grid, tile)
        M = fps.num_tiles(shape)
        packed = [torch.empty(fps.packed_bytes(shape, fps.PREC_FP8), dtype=torch.uint8, device=dev) for _ in range(3)]
        scales = [torch.empty((1, w.heads, 128 if (i == 2 and vscale == fps.VSCALE_CHANNEL) else M),
                              dtype=torch.float32, device=dev) for i in range(3)]

        def prep():
            for i in range(3):
                fps.quantize_tiles(shape, raster[i], i, vscale=vscale, out=packed[i], scales=scales[i], raster=True)

        def attn():
            fps.attn_fwd(shape, window, fps.PREC_FP8, packed[0], packed[1], packed[2], scales[0], scales[1],
                         scales[2], vscale=vscale, out=out, raster_out=True)
        prep_ms = timed(prep)
        attn_ms = timed(attn)
        return record(name, shape, tile, window, prep_ms, attn_ms, "fp8")

    def bf16_case(name, tile, window):
        shape = fps.make_shape(w.heads, w.grid, tile)
        M = fps.num_tiles(shape)
        packed = [torch.empty(fps.packed_bytes(shape, fps.PREC_BF16), dtype=torch.uint8, device=dev) for _ in range(3)]
        vs = torch.empty((1, w.heads, M), dtype=torch.float32, device=dev)

        def prep():
            for i in range(3):
                fps.pack_tiles_bf16(shape, raster[i], i, out=packed[i], vscale=vs, raster=True)

        def attn():
            fps.attn_fwd(shape, window, fps.PREC_BF16, packed[0], packed[1], packed[2], sv=vs, out=out,
                         raster_out=True)
        prep_ms = timed(prep)
        attn_ms = timed(attn)
        return record(name, shape, tile, window, prep_ms, attn_ms, "bf16")

    def record(name, shape, tile, window, prep_ms, attn_ms, prec):
        _, pairs = fps.tile_mask_host(shape, window)
        ts = tile[0] * tile[1] * tile[2]
        flop = pairs * w.heads * 4.0 * ts * ts * w.head_dim
        return {"name": name, "precision": prec, "tile": list(tile), "tile_tokens": ts,
                "tile_slots": fps.tile_slots(shape), "window": list(window), "kept_tile_pairs": pairs,
                "prepare_ms": prep_ms, "attention_ms": attn_ms,
                "attention_tflops": flop / attn_ms / 1e9, "whole_path_tflops": flop / (prep_ms + attn_ms) / 1e9}

    base, win = tuple(w.tile), tuple(w.window)
    rows = [fp8_case("per-tile V scales (the workload itself)", base, win),
            fp8_case("per-channel V scales (Sec. 3.2)", base, win, vscale=fps.VSCALE_CHANNEL),
            bf16_case("BF16 operands, same sparse window", base, win),
            fp8_case("shifted-window edge rule", base, win + (fps.EDGE_SHIFT,)),
            fp8_case("tile (2,8,16): 256 tokens, 2 blocks", (2, 8, 16), (3, 3, 3)),
            fp8_case("tile (6,8,8): 384 tokens, 3 blocks", (6, 8, 8), (1, 3, 5)),
            fp8_case("tile (3,4,4): 48 tokens in two 32-slot blocks", (3, 4, 4), (1, 7, 13)),
            fp8_case("tile (12,16,16): 3072 tokens, 24 blocks", (12, 16, 16), (1, 1, 3))]
    return rows


def run_window_ablation(dev, reps=10):
    """The window sizes (t,h,w) of the paper's window ablation (Table 4, Wan2.1-1.3B; kernel
    speed-ups 3.24x / 3.07x / 1.69x / 5.16x over BF16 on H20, tile not stated) on the 480p grid with
    the (6,8,8) tile the paper calls hardware-friendly and with the (1,8,16) tile of the other
    workloads: FP8 attention ms per call and the speed-up over this build's dense BF16 kernel."""
    import torch
    from paper_2506_04648_amd import fps, synth
    w = synth.WAN_1_3B_480P
    q, k, v = synth.qkv_raster(w, workers=min(16, os.cpu_count() or 1))
    raster = [torch.from_numpy(a[None]).to(dev).to(torch.bfloat16) for a in (q, k, v)]
    del q, k, v
    out = torch.empty((1, w.heads) + tuple(w.grid) + (128,), dtype=torch.bfloat16, device=dev)
    ev = lambda: torch.cuda.Event(enable_timing=True)

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        a, b = ev(), ev()
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    rows = []
    for tile in ((6, 8, 8), (1, 8, 16)):
        shape = fps.make_shape(w.heads, w.grid, tile)
        M = fps.num_tiles(shape)
        p16 = [fps.pack_tiles_bf16(shape, raster[i], i, raster=True) for i in range(3)]
        dense_win = tuple(2 * (-(-g // t)) - 1 for g, t in zip(w.grid, tile))
        dense_ms = timed(lambda: fps.attn_fwd(shape, dense_win, fps.PREC_BF16, p16[0][0], p16[1][0], p16[2][0],
                                              sv=p16[2][1], out=out, raster_out=True))
        del p16
        q8 = [fps.quantize_tiles(shape, raster[i], i, raster=True) for i in range(3)]
        quant_ms = timed(lambda: [fps.quantize_tiles(shape, raster[i], i, out=q8[i][0], scales=q8[i][1], raster=True)
                                  for i in range(3)])
        for window in ((3, 3, 1), (5, 6, 10), (6, 6, 6), (6, 6, 1)):
            ms = timed(lambda: fps.attn_fwd(shape, window, fps.PREC_FP8, q8[0][0], q8[1][0], q8[2][0],
                                            q8[0][1], q8[1][1], q8[2][1], out=out, raster_out=True))
            _, pairs = fps.tile_mask_host(shape, window)
            rows.append({"tile": list(tile), "window": list(window), "kept_tile_pairs": pairs, "of_pairs": M * M,
                         "fp8_attention_ms": ms, "quantize_x3_ms": quant_ms, "dense_bf16_ms": dense_ms,
                         "speedup_attention_only": dense_ms / ms, "speedup_with_quantize": dense_ms / (ms + quant_ms)})
        del q8
    return {"workload": w.name, "paper_speedups_H20": {"3,3,1": 3.24, "5,6,10": 3.07, "6,6,6": 1.69, "6,6,1": 5.16},
            "rows": rows}


def run_schedule(w, shape, dev, num_steps=50, alpha1=0.2, alpha2=0.5):
    """Denoising-step-aware schedule (Eq. 6) with the thresholds t1 = 0.2 D, t2 = 0.5 D, D = 50: calls
    1-10 dense BF16, 11-25 FP8 with a 7x5x5-tile window, 26-50 FP8 with a 3x3x3-tile window, every
    call on its own seed-generated Q, K, V (all 50 sets resident in HBM before the clock starts).
    Each call runs the whole path for its regime: FP8 = fused tile-order+quantise x3 + attention;
    BF16 = fused tile-order+operand packing x3 + attention.  The regime is picked by the library from
    the step configuration passed to fps_attn_fwd."""
    import torch
    from paper_2506_04648_amd import fps, synth
    dense_win = tuple(2 * (-(-g // t)) - 1 for g, t in zip(w.grid, w.tile))
    regimes = [(fps.PREC_BF16, dense_win), (fps.PREC_FP8, (7, 5, 5)), (fps.PREC_FP8, (3, 3, 3))]
    TS = w.tile[0] * w.tile[1] * w.tile[2]
    t0 = time.time()
    inputs = []
    for call in range(num_steps):
        q, k, v = synth.qkv_raster(w, call_index=call, workers=min(16, os.cpu_count() or 1))
        inputs.append([torch.from_numpy(a[None]).to(dev).to(torch.bfloat16) for a in (q, k, v)])
        del q, k, v
    gen_s = time.time() - t0
    M = fps.num_tiles(shape)
    L = M * fps.tile_slots(shape)
    packed8 = [torch.empty(fps.packed_bytes(shape, fps.PREC_FP8), dtype=torch.uint8, device=dev) for _ in range(3)]
    packed16 = [torch.empty(fps.packed_bytes(shape, fps.PREC_BF16), dtype=torch.uint8, device=dev) for _ in range(3)]
    scales = [torch.empty((1, w.heads, M), dtype=torch.float32, device=dev) for _ in range(3)]
    out = torch.empty((1, w.heads) + tuple(w.grid) + (128,), dtype=torch.bfloat16, device=dev)

    def call_step(step):
        cfg = fps.make_step_cfg(step, num_steps, alpha1, alpha2, regimes)
        prec, _ = fps.schedule_select(cfg)
        x = inputs[step - 1]
        if prec == fps.PREC_FP8:
            for i in range(3):
                fps.quantize_tiles(shape, x[i], i, out=packed8[i], scales=scales[i], raster=True)
            fps.attn_fwd(shape, None, prec, packed8[0], packed8[1], packed8[2], scales[0], scales[1],
                         scales[2], out=out, raster_out=True, step=cfg)
        else:
            for i in range(3):
                fps.pack_tiles_bf16(shape, x[i], i, out=packed16[i], vscale=scales[2], raster=True)
            fps.attn_fwd(shape, None, prec, packed16[0], packed16[1], packed16[2], sv=scales[2], out=out,
                         raster_out=True, step=cfg)
        return prec

    call_step(1); call_step(11); call_step(26)                 # warm-up of the three regimes
    torch.cuda.synchronize()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(num_steps + 1)]
    t0 = time.perf_counter()
    marks[0].record()
    for step in range(1, num_steps + 1):
        call_step(step)
        marks[step].record()
    torch.cuda.synchronize()
    total_ms = (time.perf_counter() - t0) * 1e3
    per_call = [marks[i].elapsed_time(marks[i + 1]) for i in range(num_steps)]
    res = {"num_steps": num_steps, "alpha": [alpha1, alpha2], "total_ms": total_ms, "input_gen_s": round(gen_s, 1),
           "regimes": []}
    bounds = [(0, 10, "dense BF16"), (10, 25, "FP8 window 7x5x5"), (25, 50, "FP8 window 3x3x3")]
    for (lo, hi, name), (prec, win) in zip(bounds, regimes):
        pairs, _ = kept_pairs(w.grid, w.tile, win)
        flop = pairs * w.heads * 4.0 * TS * TS * w.head_dim
        ms = sum(per_call[lo:hi]) / (hi - lo)
        res["regimes"].append({"calls": hi - lo, "mode": name, "window_tiles": list(win), "kept_tile_pairs": pairs,
                               "ms_per_call": ms, "tflops_whole_path": flop / ms / 1e9})
    return res


def cpu_baseline(w, n_heads, TS):
    """The oracle as it stands, timed on the host cores on a bounded sample of the same workload:
    the first n_heads heads, each in full (tile order, per-tile quantisation of Q, K, V, attention
    for every query tile).  Reported in the metric's unit on the sample's own computed tile pairs."""
    import numpy as np
    from paper_2506_04648_amd import synth
    from oracle import fps_oracle as fo
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = 1
    g = fo.Geometry(*w.grid, *w.tile)
    heads = list(range(min(n_heads, w.heads)))
    q, k, v = synth.qkv_raster(w, heads=heads)
    t0 = time.perf_counter()
    for h in range(len(heads)):
        qt, kt, vt = (fo.tile_order(a[h].astype(np.float64), g) for a in (q, k, v))
        fo.attention(qt, kt, vt, g, w.window)
    secs = time.perf_counter() - t0
    sample_pairs = int(fo.tile_mask(g, w.window).sum()) * len(heads)
    sflop = sample_pairs * 4.0 * TS * TS * w.head_dim
    total_pairs = int(fo.tile_mask(g, w.window).sum()) * w.heads
    return {"value": sflop / secs / 1e12, "unit": "TFLOP/s (computed tile pairs)", "cores": threads,
            "kind": "oracle", "seconds": secs, "sample_tile_pairs": sample_pairs,
            "extrapolated_full_call_seconds": secs * total_pairs / sample_pairs,
            "sample": f"{len(heads)} of {w.heads} heads of {w.name}, each complete: tile order + quantise all "
                      f"{g.M} tiles of Q,K,V + attention for all {g.M} query tiles ({sample_pairs} tile "
                      f"pairs); BLAS threads = cores, elementwise NumPy is single-threaded"}


if __name__ == "__main__":
    main()
