"""Prints how many shader clocks a SIMD spends per group of (one matrix instruction + n vector
instructions), with one wave on it and with two that interleave, measured with fps_debug_issue_mix:
the yardstick for the attention kernels' cycles per key block.  Run as  python -m paper_2506_04648_amd.issue_model"""
from __future__ import annotations

import sys

NV = (0, 1, 2, 4, 6, 8, 12, 16, 24, 32)
KINDS = ((0, "E4M3 16x16x128"), (3, "E4M3 32x32x64"), (1, "bf16 16x16x32"), (4, "bf16 32x32x16"), (2, "no MFMA"))


def measure(kind, nv, op, per_cu, iters=2000, cus=256, per_wave=False):
    import torch
    from . import fps
    dev = torch.device("cuda:0")
    wgs = cus * per_cu
    sink = torch.empty(wgs * 256, dtype=torch.float32, device=dev)
    cyc = torch.zeros(wgs * 4, dtype=torch.int64, device=dev)
    fps.debug_issue_mix(kind, nv, op, per_cu, wgs, iters, sink, cyc)      # warm-up
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    fps.debug_issue_mix(kind, nv, op, per_cu, wgs, iters, sink, cyc)
    b.record()
    torch.cuda.synchronize()
    if per_wave:
        c = cyc.double() / (iters * 8)
        return float(c.min()), float(c.median()), float(c.max())
    # All waves are resident from the start, and the SIMD serves the older of two waves first (the
    # younger one gets what is left), so single waves' counts say little: the longest count is the
    # launch's duration in shader clocks, and the SIMD spent it on per_cu waves' groups.
    longest = float(cyc.max())
    return longest / (iters * 8 * per_cu), longest / (a.elapsed_time(b) * 1e-3) / 1e9   # clocks per group and SIMD, GHz


def main(argv=None):
    print("SIMD clocks per group of 1 matrix instruction + n vector units; unit = one v_fma_f32 "
          "(fma) or one v_exp_f32 with one v_add_f32 (exp)")
    for op, opname in ((0, "fma"), (1, "exp")):
        for kind, kname in KINDS:
            for per_cu in (1, 2):
                row, ghz = [], 0.0
                for nv in NV:
                    if kind == 2 and nv == 0:
                        row.append("   -  ")
                        continue
                    g, ghz = measure(kind, nv, op, per_cu)
                    row.append("%6.1f" % g)
                print("%-15s %-3s waves/SIMD %d | n = %s : %s | %.2f GHz" %
                      (kname, opname, per_cu, " ".join("%d" % n for n in NV), " ".join(row), ghz), flush=True)
    lo, med, hi = measure(0, 0, 0, 2, per_wave=True)
    print("E4M3 16x16x128 alone, two waves per SIMD, clocks per instruction counted by single waves: "
          "fastest %.1f, median %.1f, slowest %.1f (the older wave of a SIMD is served first)" % (lo, med, hi))
    return 0


if __name__ == "__main__":
    sys.exit(main())
