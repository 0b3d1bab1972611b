// Device helpers shared by the data-movement kernels of libfps (not part of the ABI).
#pragma once
#include "fps_internal.h"

namespace fps {

// Where a block of BS slots sits: its head, the grid origin of its SUB-TILE and its first slot
// within the sub-tile.  Computed once per workgroup (the divisions are by run-time values).
struct BlockOrigin {
    long long bh;
    int t0, h0, w0;      // grid coordinates of the sub-tile's first token
    int slot0;           // first in-sub-tile slot of the block
};
__device__ __forceinline__ BlockOrigin block_origin(const Geom& g, int blk) {
    BlockOrigin o;
    const int group = blk / g.KBS;                       // 32-bit: the block count fits a grid dimension
    o.slot0 = (blk - group * g.KBS) * g.BS;
    const int tile_lin = group / g.NS, s = group - tile_lin * g.NS;
    const int bh = tile_lin / g.M;
    const int u = tile_lin - bh * g.M;
    const int ut = u / (g.nW * g.nH), rem = u - ut * (g.nW * g.nH);
    const int uh = rem / g.nW, uw = rem - uh * g.nW;
    const int st = s / (g.nsH * g.nsW), srem = s - st * (g.nsH * g.nsW);
    const int sh = srem / g.nsW, sw = srem - sh * g.nsW;
    o.bh = bh;
    o.t0 = ut * g.Tt + st * g.Qt; o.h0 = uh * g.Th + sh * g.Qh; o.w0 = uw * g.Tw + sw * g.Qw;
    return o;
}

// The 16 uint4 (256 bytes) of the bf16 row of the token in slot r of block `blk`.  TILED input:
// blocks are contiguous.  RASTER input: the token's (t,h,w) is recovered from the sub-tile origin
// and the in-sub-tile slot; padding slots return nullptr.
template <bool RASTER>
__device__ __forceinline__ const uint4* token_row(const uint4* x, const Geom& g, const BlockOrigin& o,
                                                  int blk, int r) {
    if (!RASTER) return x + ((long long)blk * g.BS + r) * 16;
    const int slot = o.slot0 + r;
    if (slot >= g.QS) return nullptr;                    // slots past the sub-tile's tokens are padding
    const int rt = div_by_recip(slot, g.inv_qplane), rem = slot - rt * (g.Qh * g.Qw);
    const int rh = div_by_recip(rem, g.inv_qw), rw = rem - rh * g.Qw;
    const int t = o.t0 + rt, h = o.h0 + rh, w = o.w0 + rw;
    if (t >= g.T || h >= g.H || w >= g.W) return nullptr;
    return x + ((((o.bh * g.T + t) * g.H + h) * (long long)g.W + w) * 16);
}

// max of the 15-bit magnitude patterns of 8 bf16 values (|x| of bf16 orders like that integer),
// two patterns per instruction: the running maximum m2 holds one candidate in each 16-bit half
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t amax_pairs16(const uint4& v, uint32_t m2) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    u16x2 m = __builtin_bit_cast(u16x2, m2);
#pragma unroll
    for (int i = 0; i < 4; ++i) m = __builtin_elementwise_max(m, __builtin_bit_cast(u16x2, w[i] & 0x7FFF7FFFu));
    return __builtin_bit_cast(uint32_t, m);
}
__device__ __forceinline__ uint32_t amax_of_pairs(uint32_t m2) {        // the larger half
    const uint32_t lo = m2 & 0xFFFFu, hi = m2 >> 16;
    return lo > hi ? lo : hi;
}
__device__ __forceinline__ uint32_t amax_bits16(const uint4& v, uint32_t m) {
    const uint32_t p = amax_of_pairs(amax_pairs16(v, 0u));
    return p > m ? p : m;
}

// workgroup-wide max of m over 256 threads (red: 4 words of LDS); every thread gets the result
__device__ __forceinline__ uint32_t block_max_256(uint32_t m, uint32_t* red) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const uint32_t o = (uint32_t)__shfl_xor((int)m, off);
        m = o > m ? o : m;
    }
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
    __syncthreads();
    m = red[0];
#pragma unroll
    for (int i = 1; i < 4; ++i) m = red[i] > m ? red[i] : m;
    return m;
}

__device__ __forceinline__ int pow2_exponent_for_fp16(float amax) {   // e with amax*2^-e in [2^14,2^15)
    const uint32_t bits = __float_as_uint(amax);
    int e = (int)((bits >> 23) & 0xFF) - 127 - 14;
    return bits == 0 ? 0 : (e < -100 ? -100 : (e > 113 ? 113 : e));
}

// small in-place helpers (static: each translation unit that launches them has its own copy)
static __global__ void clear_kernel(uint32_t* p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}
static __global__ void amax_to_scale_kernel(float* p, int n) {       // amax -> amax/448 (1 for 0)
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) { const float a = p[i]; p[i] = a == 0.0f ? 1.0f : a / 448.0f; }
}
static __global__ void amax_to_pow2_kernel(float* p, int n) {        // amax -> 2^e (see above)
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = __uint_as_float((uint32_t)(127 + pow2_exponent_for_fp16(p[i])) << 23);
}
// amax over the KBS blocks of each quantisation group: one workgroup per block, merged with an
// atomic max on the float bit pattern (amax_bits must be cleared first)
template <bool RASTER>
__global__ __launch_bounds__(256) void block_amax_kernel(const uint4* __restrict__ x,
                                                         uint32_t* __restrict__ amax_bits, Geom g) {
    __shared__ uint32_t red[4];
    uint32_t m = 0;
    const BlockOrigin org = block_origin(g, blockIdx.x);
    for (int c = threadIdx.x; c < g.BS * 16; c += 256) {
        const uint4* row = token_row<RASTER>(x, g, org, blockIdx.x, c >> 4);
        if (row) m = amax_bits16(row[c & 15], m);
    }
    m = block_max_256(m, red);
    if (threadIdx.x == 0) atomicMax(&amax_bits[blockIdx.x / g.KBS], m << 16);
}

}  // namespace fps
