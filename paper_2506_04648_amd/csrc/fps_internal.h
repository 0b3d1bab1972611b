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
    // The kernels work on blocks of BS tokens (128 or 32); a tile occupies KB = ceil(TS/BS)
    // consecutive blocks, TSP = KB*BS slots, and has ONE scale.  Block index = tile * KB + block
    // in tile.  Slot r of a tile holds the token of in-tile rank r if r < TS, else padding.
    int BS, KB, TSP;
    // Real planes / rows / columns of the LAST tile along each axis (all others are full).  A
    // tile's boundary class is c = 4*(last along T) + 2*(last along H) + (last along W).
    int lastT, lastH, lastW;
    // Blocks of a last-along-T tile that hold at least one real token: its slots from
    // lastT*Th*Tw on are all padding, so those blocks are never computed.
    int kb_last;
};

// slot r of a tile of boundary class c holds a real token
__host__ __device__ inline bool slot_is_token(const Geom& g, int c, int r) {
    if (r >= g.TS) return false;
    const int plane = g.Th * g.Tw;
    const int rt = r / plane, rem = r - rt * plane;
    const int rh = rem / g.Tw, rw = rem - rh * g.Tw;
    return rt < ((c & 4) ? g.lastT : g.Tt) && rh < ((c & 2) ? g.lastH : g.Th) &&
           rw < ((c & 1) ? g.lastW : g.Tw);
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
int launch_pack_bf16(const Geom& g, const void* x, int role, void* xp, float* vscale, hipStream_t st);
int launch_unpack_q8(const Geom& g, const void* xq, int role, uint8_t* out, hipStream_t st);
int launch_attn(const Geom& g, const fps_window& win, int prec, const void* q, const void* k,
                const void* v, const float* sq, const float* sk, const float* sv, int vscale,
                void* out, int out_f32, int out_raster, uint8_t* visited, hipStream_t st);

int launch_copy(const void* in, void* out, long long bytes, hipStream_t st);
int launch_scores_fp8(const Geom& g, const void* q, const void* k, int bh, int u, int v, float* out,
                      hipStream_t st);
int launch_scores_block_fp8(const Geom& g, const void* q, const void* k, int bh, int u, int jq, int v,
                            int jk, float* out, hipStream_t st);

}  // namespace fps
