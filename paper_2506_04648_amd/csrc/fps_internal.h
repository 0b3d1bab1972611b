// Internal declarations shared by the translation units of libfps (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdarg.h>
#include "fps.h"

namespace fps {

constexpr int kHeadDim = 128;
constexpr int kMaxTileTokens = 32768;                // largest supported tile
constexpr int kMaxScoreSlots = 4096;                 // largest tile the score debug call accepts

// Everything the kernels derive from an fps_shape.
struct Geom {
    int BH;              // B * heads
    int T, H, W;
    int Tt, Th, Tw;
    int nT, nH, nW;
    int M, TS;
    // Quantisation sub-tile (Qt,Qh,Qw) (= the tile when none is given): a tile is NS = nsT*nsH*nsW
    // sub-tiles of QS tokens, each with its own scale; sub-tile s = (st*nsH + sh)*nsW + sw.
    int Qt, Qh, Qw;
    int nsT, nsH, nsW, NS, QS;
    float inv_qplane, inv_qw;   // 1/(Qh*Qw) and 1/Qw as correctly rounded floats, for div_by_recip
    // The kernels work on blocks of BS slots (128 or 32).  A sub-tile occupies KBS = ceil(QS/BS)
    // consecutive blocks (QSP = KBS*BS slots, slot rr < QS holding the token of in-sub-tile rank
    // rr, the rest padding), a tile KB = NS*KBS blocks (TSP = KB*BS slots).  Block index =
    // tile * KB + block in tile; scale (group) index = tile * NS + sub-tile = block index / KBS.
    int BS, KBS, QSP, KB, TSP;
    // Real planes / rows / columns of the LAST tile along each axis (all others are full).  A
    // tile's boundary class is c = 4*(last along T) + 2*(last along H) + (last along W).
    int lastT, lastH, lastW;
    // Leading blocks of a last-along-T tile that can hold a real token: the blocks after them
    // are padding only and are never computed.
    int kb_last;
};

// n / d for 0 <= n < 2^21, given inv_d = 1.0f / d correctly rounded.  Exact: (n + 1/2) / d is at
// least 1/(2d) away from every integer, and the float product errs by less than n 2^-22 / d.
// Four cheap instructions instead of the ~25 of an integer division by a run-time value.
__host__ __device__ inline int div_by_recip(int n, float inv_d) {
    return (int)(((float)n + 0.5f) * inv_d);
}

// In-tile coordinates of the first token of sub-tile s (decoded once per block: s is the same
// for all slots of a block).
struct SubTile { int t0, h0, w0; };
__host__ __device__ inline SubTile sub_tile_origin(const Geom& g, int s) {
    const int layer = g.nsH * g.nsW;
    const int st = s / layer, srem = s - st * layer;
    const int sh = srem / g.nsW, sw = srem - sh * g.nsW;
    return SubTile{st * g.Qt, sh * g.Qh, sw * g.Qw};
}

// In-tile coordinates (rt, rh, rw) of slot rr of the sub-tile with origin o; false if the slot is
// padding of the sub-tile (rr >= QS).
__host__ __device__ inline bool sub_slot_coords(const Geom& g, const SubTile& o, int rr, int* rt, int* rh, int* rw) {
    if (rr >= g.QS) return false;
    const int a = div_by_recip(rr, g.inv_qplane), rem = rr - a * (g.Qh * g.Qw);
    const int b = div_by_recip(rem, g.inv_qw), c = rem - b * g.Qw;
    *rt = o.t0 + a; *rh = o.h0 + b; *rw = o.w0 + c;
    return true;
}

// in-tile coordinates (rt, rh, rw) lie inside the real extent of a tile of boundary class c
__host__ __device__ inline bool coords_in_class(const Geom& g, int c, int rt, int rh, int rw) {
    return rt < ((c & 4) ? g.lastT : g.Tt) && rh < ((c & 2) ? g.lastH : g.Th) &&
           rw < ((c & 1) ? g.lastW : g.Tw);
}

// slot rr of the sub-tile with origin o, in a tile of boundary class c, holds a real token
__host__ __device__ inline bool sub_slot_is_token(const Geom& g, int c, const SubTile& o, int rr) {
    int rt, rh, rw;
    return sub_slot_coords(g, o, rr, &rt, &rh, &rw) && coords_in_class(g, c, rt, rh, rw);
}

// slot r (0 .. TSP-1) of a tile of boundary class c holds a real token
__host__ __device__ inline bool slot_is_token(const Geom& g, int c, int r) {
    const int s = r / g.QSP;
    return sub_slot_is_token(g, c, sub_tile_origin(g, s), r - s * g.QSP);
}

void set_error(const char* fmt, ...);
int check_shape(const fps_shape* s, Geom* g);          // validates, fills g
int check_ptr(const void* p, const char* name);        // non-null and 16-byte aligned
int hip_fail(hipError_t e, const char* what);          // records and returns FPS_ERR_HIP

// kernel launchers (defined in the .hip files); all arguments already validated
int launch_tile_order(const Geom& g, const void* in, void* out, hipStream_t st);
int launch_tile_unorder(const Geom& g, const void* in, int elem_bytes, void* out, hipStream_t st);
int launch_quantize(const Geom& g, const void* x, int raster, int role, int vscale, void* xq,
                    float* scales, hipStream_t st);
int launch_pack_bf16(const Geom& g, const void* x, int raster, int role, void* xp, float* vscale,
                     hipStream_t st);
int launch_unpack_q8(const Geom& g, const void* xq, int role, uint8_t* out, hipStream_t st);
int launch_attn(const Geom& g, const fps_window& win, int prec, const void* q, const void* k,
                const void* v, const float* sq, const float* sk, const float* sv, int vscale,
                void* out, int out_f32, int out_raster, uint8_t* visited, hipStream_t st);

int launch_copy(const void* in, void* out, long long bytes, hipStream_t st);
int launch_mfma_rate(int workgroups, int iters, float* sink, hipStream_t st);
int launch_issue_mix(int kind, int nv, int op, int workgroups_per_cu, int workgroups, int iters,
                     float* sink, unsigned long long* cycles, hipStream_t st);
int launch_scores_fp8(const Geom& g, const void* q, const void* k, int bh, int u, int v, float* out,
                      hipStream_t st);
int launch_scores_block_fp8(const Geom& g, const void* q, const void* k, int bh, int u, int jq, int v,
                            int jk, float* out, hipStream_t st);

}  // namespace fps
