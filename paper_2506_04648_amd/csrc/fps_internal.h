// Internal declarations shared by the translation units of libfps (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdarg.h>
#include "fps.h"

namespace fps {

constexpr int kHeadDim = 128;
constexpr int kMaxTileTokens = 1024;                 // largest supported tile
constexpr int kMaxTileWords = kMaxTileTokens / 32;

// Everything the kernels derive from an fps_shape.
struct Geom {
    int BH;              // B * heads
    int T, H, W;
    int Tt, Th, Tw;
    int nT, nH, nW;
    int M, TS;
    // The kernels work on blocks of BS tokens (128, or 32 for 32-token tiles); a tile is KB = TS/BS
    // consecutive blocks that share one scale.  Block index = tile index * KB + block in tile.
    int BS, KB;
    // valid_mask[c][w]: bit (r & 31) of word (r >> 5) is set iff the token of in-tile rank r is a
    // real token in a tile of boundary class c = 4*(last tile along T) + 2*(last along H) +
    // (last along W).  A tile that is last along an axis keeps only T - (nT-1)*Tt (etc.) planes.
    uint32_t valid_mask[8][kMaxTileWords];
};

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

}  // namespace fps
