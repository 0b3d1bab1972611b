// Per-group amax -> scale -> E4M3 encode (Sec. 3.2, Eq. 4-5; Algorithm 1 step 2), writing the
// packed operand layouts described in fps_layout.hip.  A scale group is a 3D tile, or a
// quantisation sub-tile of it.  One workgroup of 256 threads per block of BS slots; the pass is
// HBM-bound (2 bytes read, 1 byte written per element).
#include "fps_device_common.h"

namespace fps {

__device__ __forceinline__ int key_of_slot_q(int g, int s) { return 16 * (s >> 2) + 4 * g + (s & 3); }
// 128-slot blocks (32x32x64 MFMA): the key behind byte jj of 16-byte half e of contraction step j in
// lane half h -- where the accumulator of S^T = K Q^T left that key's weight
__device__ __forceinline__ int key_of_slot_wide(int j, int e, int h, int jj) {
    return 32 * (2 * j + e) + 8 * (jj >> 2) + 4 * h + (jj & 3);
}

// Quotient x/s prepared for the hardware's round-to-nearest-even conversion so that the final code
// equals the rounding of the EXACT quotient: the correctly rounded float quotient can land exactly
// on an E4M3 rounding midpoint although the true quotient lies beside it; the sign of the exact
// residual x - q*s (one fma) tells on which side, and q is moved one float ulp that way.
__device__ __forceinline__ float quotient_for_rne(float x, float s) {
    float q = x / s;
    uint32_t qb = __float_as_uint(q);
    const float a = __builtin_fabsf(q);
    bool mid;
    if (a >= 0.015625f) {
        mid = (qb & 0xFFFFFu) == 0x80000u;          // 3 mantissa bits kept, next bit set, rest zero
    } else {
        const float t = a * 1024.0f;                 // subnormal grid 2^-9: midpoints are odd * 2^-10
        mid = (t == __builtin_floorf(t)) && (((int)t) & 1);
    }
    if (mid) {
        const float r = __builtin_fmaf(-q, s, x);
        if (r != 0.0f) {
            const bool up = (r > 0.0f) == (q > 0.0f);
            qb = up ? qb + 1u : qb - 1u;             // magnitude one ulp up / down
            q = __uint_as_float(qb);
        }
    }
    return __builtin_fminf(__builtin_fmaxf(q, -448.0f), 448.0f);
}

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// Same result as quotient_for_rne(x, s), cheaper on the common path: x * (1/s) is within three
// float ulps of the exact quotient, so the rounding can only differ when an E4M3 midpoint lies
// within a few ulps of the product; only then (and in the subnormal range of the format, where
// the grid is absolute) the exact routine runs.  rs = 1/s, correctly rounded.
// The product is formed as fma(x, 1/s, tiny): a zero input (padding, common) then gives `tiny`,
// which encodes as 0 like the exact path would, without taking that path; for non-zero inputs the
// addend is far below an ulp.  No clamp is needed on the common path: |x| <= amax makes the
// product at most 448 (1 + 2^-22), far below the next rounding boundary (464).
__device__ __forceinline__ float quotient_fast(float x, float s, float rs) {
    const float q = __builtin_fmaf(x, rs, 1.3e-30f);
    const uint32_t qb = __float_as_uint(q);
    const uint32_t low = (qb & 0xFFFFFu) - (0x80000u - 4u);          // distance to a midpoint pattern
    const bool near_mid = low <= 8u;
    // 2^-90 <= |q| < 2^-6 (below 2^-90, which includes `tiny`, the code is 0 either way)
    const bool subnormal = ((qb << 1) - 0x25000000u) < (0x79000000u - 0x25000000u);
    if (__builtin_expect(near_mid || subnormal, 0)) return quotient_for_rne(x, s);
    return q;
}

// 16 bf16 (two uint4) -> 16 E4M3 codes (one uint4)
__device__ __forceinline__ uint4 encode16(const uint4& lo, const uint4& hi, float s) {
    const uint32_t w[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
    const float rs = 1.0f / s;
    uint32_t o[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int r = 0;
        r = __builtin_amdgcn_cvt_pk_fp8_f32(quotient_fast(bf16_lo(w[2 * i]), s, rs),
                                            quotient_fast(bf16_hi(w[2 * i]), s, rs), r, false);
        r = __builtin_amdgcn_cvt_pk_fp8_f32(quotient_fast(bf16_lo(w[2 * i + 1]), s, rs),
                                            quotient_fast(bf16_hi(w[2 * i + 1]), s, rs), r, true);
        o[i] = (uint32_t)r;
    }
    return make_uint4(o[0], o[1], o[2], o[3]);
}

// V block in LDS (row-major codes [token][128]) -> key-contiguous packed layout in HBM
template <int BS>
__device__ __forceinline__ void write_v_block(const uint8_t* stage, uint4* dst, int tid) {
    if (BS == 128) {
        for (int c = tid; c < BS * 8; c += 256) {
            const int lane = c & 63, e = (c >> 6) & 1, j = (c >> 7) & 1, db = c >> 8;
            const int h = lane >> 5, n = lane & 31;
            union { uint4 v; uint8_t b[16]; } o;
#pragma unroll
            for (int jj = 0; jj < 16; ++jj)
                o.b[jj] = stage[key_of_slot_wide(j, e, h, jj) * 128 + 32 * db + n];
            dst[c] = o.v;
        }
    } else {
        uint2* dst8 = reinterpret_cast<uint2*>(dst);
        for (int c = tid; c < BS * 16; c += 256) {
            const int lane = c & 63, cb = c >> 6;
            const int gg = lane >> 4, n = lane & 15;
            union { uint2 v; uint8_t e[8]; } o;
#pragma unroll
            for (int jj = 0; jj < 8; ++jj)
                o.e[jj] = stage[key_of_slot_q(gg, jj) * 128 + 16 * cb + n];
            dst8[c] = o.v;
        }
    }
}

// One workgroup of 256 threads per NB consecutive blocks of BS slots.  A scale group of up to three
// blocks is handled by one workgroup in a single pass over HBM (NB = blocks per group): all its
// blocks are held in registers while the amax is reduced, then encoded.  Larger groups take their
// amax from block_amax_kernel (tile_amax != nullptr, NB = 1) and this kernel only encodes.
// RASTER: x is the raster tensor [BH,T,H,W,128] and the block's tokens are gathered from it (padded
// slots read as zero), which fuses the tile ordering of Sec. 3.2 step (1) into this pass.
template <int BS, bool RASTER, int NB>
__global__ __launch_bounds__(256) void quantize_tiles_kernel(const uint4* __restrict__ x,
                                                             uint8_t* __restrict__ xq,
                                                             float* __restrict__ scales, int role,
                                                             Geom g, const float* __restrict__ tile_amax) {
    constexpr int U = BS / 32;                      // 32-byte units (16 channels of one token) per thread
    __shared__ uint32_t red[4];
    __shared__ __attribute__((aligned(16))) uint8_t stage[BS * 128];
    const int first = blockIdx.x * NB;              // first block of this workgroup
    const int tid = threadIdx.x;

    uint4 lo[NB][U], hi[NB][U];
    uint32_t mb = 0;
#pragma unroll
    for (int kb = 0; kb < NB; ++kb) {
        const BlockOrigin org = block_origin(g, first + kb);
#pragma unroll
        for (int i = 0; i < U; ++i) {
            const int unit = tid + 256 * i;          // token = unit >> 3, 16-channel group = unit & 7
            const uint4* row = token_row<RASTER>(x, g, org, first + kb, unit >> 3);
            lo[kb][i] = make_uint4(0, 0, 0, 0);
            hi[kb][i] = lo[kb][i];
            if (row) { lo[kb][i] = row[2 * (unit & 7)]; hi[kb][i] = row[2 * (unit & 7) + 1]; }
            mb = amax_pairs16(lo[kb][i], mb);
            mb = amax_pairs16(hi[kb][i], mb);
        }
    }
    mb = amax_of_pairs(mb);
    float amax;
    if (tile_amax) {
        amax = tile_amax[first / g.KBS];
    } else {
        mb = block_max_256(mb, red);
        amax = __uint_as_float(mb << 16);
    }
    const float s = (amax == 0.0f) ? 1.0f : amax / 448.0f;   // Eq. 4 (correctly rounded division)
    if (!tile_amax && tid == 0) scales[blockIdx.x] = s;       // the workgroup is the whole group

#pragma unroll
    for (int kb = 0; kb < NB; ++kb) {
        uint4* dst = reinterpret_cast<uint4*>(xq + (long long)(first + kb) * (BS * 128));
#pragma unroll
        for (int i = 0; i < U; ++i) {
            const int unit = tid + 256 * i;
            const uint4 codes = encode16(lo[kb][i], hi[kb][i], s);
            const int j = unit >> 3, c16 = unit & 7;
            if (role == FPS_ROLE_Q) {
                dst[unit] = codes;
            } else if (role == FPS_ROLE_K) {
                if (BS == 128) {                     // 32x32x64 operand: lane 32h + n, k-step ks, 16-byte half e
                    const int kb = j >> 5, n = j & 31, ks = c16 >> 2, h = (c16 >> 1) & 1, e = c16 & 1;
                    dst[((kb * 2 + ks) * 2 + e) * 64 + 32 * h + n] = codes;
                } else {
                    const int b = j >> 4, n = j & 15, gg = c16 >> 1, h = c16 & 1;
                    dst[(b * 2 + h) * 64 + gg * 16 + n] = codes;
                }
            } else {
                reinterpret_cast<uint4*>(stage)[unit] = codes;
            }
        }
        if (role == FPS_ROLE_V) {                    // uniform branch: role is a kernel argument
            __syncthreads();
            write_v_block<BS>(stage, dst, tid);
            if (kb + 1 < NB) __syncthreads();        // the staging buffer is reused by the next block
        }
    }
}

// ---- per-channel V (Sec. 3.2, Algorithm 1 step 3): s_c = max over ALL tokens of |V[:,c]| / 448 ----
// Stream-ordered kernels: clear the 128 per-head maxima; column maxima of every block merged with
// an atomic max on the bit pattern (|x| of a float orders like its unsigned pattern); encode every
// block with the per-channel scales; finally turn the stored maxima into scales in place.
// one workgroup of 256 threads per block: thread = (token group tid/16, 8-channel chunk tid%16)
template <bool RASTER>
__global__ __launch_bounds__(256) void channel_amax_kernel(const uint4* __restrict__ x,
                                                           uint32_t* __restrict__ amax_bits, Geom g) {
    __shared__ uint32_t col[128];
    const int tid = threadIdx.x, c8 = tid & 15;
    if (tid < 128) col[tid] = 0u;
    __syncthreads();
    uint32_t m[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    const BlockOrigin org = block_origin(g, blockIdx.x);
    for (int r = tid >> 4; r < g.BS; r += 16) {
        const uint4* row = token_row<RASTER>(x, g, org, blockIdx.x, r);
        if (!row) continue;
        const uint4 v = row[c8];
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t lo = w[i] & 0x7FFFu, hi = (w[i] >> 16) & 0x7FFFu;
            m[2 * i] = lo > m[2 * i] ? lo : m[2 * i];
            m[2 * i + 1] = hi > m[2 * i + 1] ? hi : m[2 * i + 1];
        }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) atomicMax(&col[c8 * 8 + i], m[i]);
    __syncthreads();
    const long long bh = blockIdx.x / ((long long)g.M * g.KB);
    if (tid < 128) atomicMax(&amax_bits[bh * 128 + tid], col[tid] << 16);
}

template <int BS, bool RASTER>
__global__ __launch_bounds__(256) void quantize_channels_kernel(const uint4* __restrict__ x,
                                                                uint8_t* __restrict__ xq,
                                                                const float* __restrict__ amax, Geom g) {
    __shared__ __attribute__((aligned(16))) uint8_t stage[BS * 128];
    __shared__ float sc[128];
    const int tid = threadIdx.x;
    const long long blk = blockIdx.x;
    const long long bh = blk / ((long long)g.M * g.KB);
    if (tid < 128) {
        const float a = amax[bh * 128 + tid];
        sc[tid] = a == 0.0f ? 1.0f : a / 448.0f;
    }
    __syncthreads();
    const BlockOrigin org = block_origin(g, blockIdx.x);
    for (int unit = tid; unit < BS * 8; unit += 256) {       // 16 channels of one token
        const int r = unit >> 3, c16 = unit & 7;
        const uint4* row = token_row<RASTER>(x, g, org, blockIdx.x, r);
        uint4 lo = make_uint4(0, 0, 0, 0), hi = lo;
        if (row) { lo = row[2 * c16]; hi = row[2 * c16 + 1]; }
        const uint32_t w[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
        uint32_t o[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float* s4 = &sc[c16 * 16 + 4 * i];
            int rr = 0;
            rr = __builtin_amdgcn_cvt_pk_fp8_f32(quotient_for_rne(bf16_lo(w[2 * i]), s4[0]),
                                                 quotient_for_rne(bf16_hi(w[2 * i]), s4[1]), rr, false);
            rr = __builtin_amdgcn_cvt_pk_fp8_f32(quotient_for_rne(bf16_lo(w[2 * i + 1]), s4[2]),
                                                 quotient_for_rne(bf16_hi(w[2 * i + 1]), s4[3]), rr, true);
            o[i] = (uint32_t)rr;
        }
        reinterpret_cast<uint4*>(stage)[unit] = make_uint4(o[0], o[1], o[2], o[3]);
    }
    __syncthreads();
    write_v_block<BS>(stage, reinterpret_cast<uint4*>(xq + blk * (BS * 128)), tid);
}

static int launch_quantize_channels(const Geom& g, const void* x, int raster, void* xq, float* scales,
                                    hipStream_t st) {
    const int blocks = g.BH * g.M * g.KB, n = g.BH * 128;
    const uint4* xi = (const uint4*)x;
    uint8_t* xo = (uint8_t*)xq;
    clear_kernel<<<(n + 255) / 256, 256, 0, st>>>((uint32_t*)scales, n);
    if (raster) channel_amax_kernel<true><<<blocks, 256, 0, st>>>(xi, (uint32_t*)scales, g);
    else        channel_amax_kernel<false><<<blocks, 256, 0, st>>>(xi, (uint32_t*)scales, g);
    if (g.BS == 128) {
        if (raster) quantize_channels_kernel<128, true><<<blocks, 256, 0, st>>>(xi, xo, scales, g);
        else        quantize_channels_kernel<128, false><<<blocks, 256, 0, st>>>(xi, xo, scales, g);
    } else {
        if (raster) quantize_channels_kernel<32, true><<<blocks, 256, 0, st>>>(xi, xo, scales, g);
        else        quantize_channels_kernel<32, false><<<blocks, 256, 0, st>>>(xi, xo, scales, g);
    }
    amax_to_scale_kernel<<<(n + 255) / 256, 256, 0, st>>>(scales, n);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? FPS_OK : hip_fail(e, "quantize_channels launch");
}

template <int BS, int NB>
static void launch_quantize_nb(const Geom& g, const uint4* xi, int raster, int role, uint8_t* xo, float* scales,
                               const float* tile_amax, int grid, hipStream_t st) {
    if (raster) quantize_tiles_kernel<BS, true, NB><<<grid, 256, 0, st>>>(xi, xo, scales, role, g, tile_amax);
    else        quantize_tiles_kernel<BS, false, NB><<<grid, 256, 0, st>>>(xi, xo, scales, role, g, tile_amax);
}

int launch_quantize(const Geom& g, const void* x, int raster, int role, int vscale, void* xq,
                    float* scales, hipStream_t st) {
    if (vscale != FPS_VSCALE_TILE) return launch_quantize_channels(g, x, raster, xq, scales, st);
    const int blocks = g.BH * g.M * g.KB, groups = g.BH * g.M * g.NS;
    const uint4* xi = (const uint4*)x;
    uint8_t* xo = (uint8_t*)xq;
    if (g.KBS <= 3) {                   // one workgroup per scale group: a single pass over the input
        if (g.BS == 128) {
            switch (g.KBS) {
                case 1: launch_quantize_nb<128, 1>(g, xi, raster, role, xo, scales, nullptr, groups, st); break;
                case 2: launch_quantize_nb<128, 2>(g, xi, raster, role, xo, scales, nullptr, groups, st); break;
                default: launch_quantize_nb<128, 3>(g, xi, raster, role, xo, scales, nullptr, groups, st); break;
            }
        } else {                        // 32-slot blocks: groups of at most 96 tokens, three blocks
            switch (g.KBS) {
                case 1: launch_quantize_nb<32, 1>(g, xi, raster, role, xo, scales, nullptr, groups, st); break;
                case 2: launch_quantize_nb<32, 2>(g, xi, raster, role, xo, scales, nullptr, groups, st); break;
                default: launch_quantize_nb<32, 3>(g, xi, raster, role, xo, scales, nullptr, groups, st); break;
            }
        }
    } else {                            // group amax over many blocks first; `scales` holds it meanwhile
        clear_kernel<<<(groups + 255) / 256, 256, 0, st>>>((uint32_t*)scales, groups);
        if (raster) block_amax_kernel<true><<<blocks, 256, 0, st>>>(xi, (uint32_t*)scales, g);
        else        block_amax_kernel<false><<<blocks, 256, 0, st>>>(xi, (uint32_t*)scales, g);
        launch_quantize_nb<128, 1>(g, xi, raster, role, xo, scales, scales, blocks, st);
        amax_to_scale_kernel<<<(groups + 255) / 256, 256, 0, st>>>(scales, groups);
    }
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? FPS_OK : hip_fail(e, "quantize_tiles launch");
}

}  // namespace fps
