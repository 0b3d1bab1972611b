// Layout kernels of libfps: raster <-> tile order (Sec. 3.2 step (1)), the BF16 operand packing,
// and the debug unpacking of packed E4M3 tensors.  All of them are pure data movement.
//
// Packed operand layouts, per block of BS = 128 or 32 slots (a tile is one or several blocks).
// E4M3, BS = 128 -- operands of v_mfma_f32_32x32x64_f8f6f4; lane = 32h + n, n the row of the 32-row
// operand block, h the half of the 64 contraction slots of one step:
//   Q : row-major [token][128]                                              (BS*128 bytes)
//   K : 16-byte chunk (((kb*2 + ks)*2 + e)*64 + lane) = K[32kb + n][64ks + 32h + 16e + 0..15]
//   V : 16-byte chunk (((db*2 + j)*2 + e)*64 + lane), byte jj = V[key][32db + n] with
//       key = 32(2j + e) + 8(jj/4) + 4h + jj%4
//   The accumulator of S^T = K Q^T for key block kb holds, in lane (n,h) and register r, query n and
//   key 32kb + 8(r/4) + 4h + r%4; the 32 weights of key blocks 2j and 2j+1 of a lane are therefore,
//   unchanged, its 32 contraction slots of step j of the PV product O^T = V^T P^T.
// E4M3, BS = 32 -- operands of the 16x16 instructions; lane = 16g + n:
//   Q : row-major [token][128]
//   K : 16-byte chunk ((b*2 + h)*64 + lane) = K[16b + n][32g + 16h + 0..15]
//   V :  8-byte chunk (cb*64 + lane), byte j = V[key(g,j)][16cb + n], key(g,s) = 16*(s/4) + 4g + s%4
// BF16, BS = 128 -- operands of the 32x32x16 instructions; lane = 32h + n:
//   Q : row-major [token][128]                                              (BS*256 bytes)
//   K : 16-byte chunk ((kb*8 + ks)*64 + lane) = K[32kb + n][16ks + 8h + 0..7]
//   V : 16-byte chunk ((db*8 + kk)*64 + lane), element el = V[key][32db + n] with
//       key = 32(kk/2) + 8(2(kk%2) + el/4) + 4h + el%4 (the key order of the 32x32 accumulator),
//       stored as fp16 after an exact power-of-two scaling per scale group (see pack_bf16_kernel)
// BF16, BS = 32 -- 16x16x32 instructions; lane = 16g + n:
//   Q : row-major [token][128]
//   K : 16-byte chunk ((b*4 + ks)*64 + lane) = K[16b + n][32ks + 8g + 0..7]
//   V : 16-byte chunk ((kk*8 + cb)*64 + lane), element e -> V[32kk + key(g,e)][16cb + n], fp16 as above
// key(g,s) is the key that slot s of lane group g holds after a 16x16 MFMA wrote S^T = K Q^T: the
// accumulator of lane (n,g) for key block b has keys 16b + 4g + 0..3, so P^T can be fed back as
// the second operand of the PV product without any cross-lane movement.
#include "fps_device_common.h"

namespace fps {

__device__ __forceinline__ int key_of_slot(int g, int s) { return 16 * (s >> 2) + 4 * g + (s & 3); }

// ---- raster -> tiled (bf16, 16-byte chunks of 8 channels) -------------------------------------
__global__ void tile_order_kernel(const uint4* __restrict__ in, uint4* __restrict__ out, Geom g,
                                  long long n_chunks) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_chunks) return;
    const int c16 = (int)(i & 15);
    const long long pos = i >> 4;                       // bh * (M*TSP) + u*TSP + r
    const int r = (int)(pos % g.TSP);
    const long long bu = pos / g.TSP;
    const int u = (int)(bu % g.M);
    const long long bh = bu / g.M;
    const int uw = u % g.nW, uh = (u / g.nW) % g.nH, ut = u / (g.nW * g.nH);
    const int s = r / g.QSP;
    int rt = 0, rh = 0, rw = 0;
    const bool slot_used = sub_slot_coords(g, sub_tile_origin(g, s), r - s * g.QSP, &rt, &rh, &rw);
    const int t = ut * g.Tt + rt, h = uh * g.Th + rh, w = uw * g.Tw + rw;
    uint4 val = make_uint4(0, 0, 0, 0);
    if (slot_used && t < g.T && h < g.H && w < g.W) {
        const long long src = (((bh * g.T + t) * g.H + h) * (long long)g.W + w) * 16 + c16;
        val = in[src];
    }
    out[i] = val;
}

// ---- tiled -> raster (elem_bytes 2 or 4; 16-byte chunks) ---------------------------------------
__global__ void tile_unorder_kernel(const uint4* __restrict__ in, uint4* __restrict__ out, Geom g,
                                    int chunks_per_row, long long n_chunks) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_chunks) return;
    const int c = (int)(i % chunks_per_row);
    long long tok = i / chunks_per_row;                 // ((bh*T + t)*H + h)*W + w
    const int w = (int)(tok % g.W); tok /= g.W;
    const int h = (int)(tok % g.H); tok /= g.H;
    const int t = (int)(tok % g.T);
    const long long bh = tok / g.T;
    const int u = ((t / g.Tt) * g.nH + h / g.Th) * g.nW + w / g.Tw;
    const int rt = t % g.Tt, rh = h % g.Th, rw = w % g.Tw;
    const int s = ((rt / g.Qt) * g.nsH + rh / g.Qh) * g.nsW + rw / g.Qw;
    const int r = s * g.QSP + ((rt % g.Qt) * g.Qh + rh % g.Qh) * g.Qw + rw % g.Qw;
    const long long src = ((bh * g.M + u) * (long long)g.TSP + r) * chunks_per_row + c;
    out[i] = in[src];
}

// ---- BF16 operand packing -----------------------------------------------------------------------
// One workgroup of 256 threads per block of BS tokens; the block (BS*256 bytes) is staged in LDS.
// Q and K keep their bf16 values.  V is converted to fp16 so that the PV product can take P in
// fp16 (11 significant bits instead of bf16's 8): each TILE is first multiplied by 2^-e with
// amax * 2^-e in [2^14, 2^15), which keeps every bf16 value exact unless it is more than 2^28
// times smaller than the tile's largest one, and vscale[tile] = 2^e undoes it in the kernel.
// For tiles of several blocks the tile amax is computed beforehand (tile_amax != nullptr).
// RASTER: `in` is the raster tensor and the block's tokens are gathered from it (padding slots read
// as zero), which fuses the tile ordering into this pass.
template <int BS, bool RASTER>
__global__ __launch_bounds__(256) void pack_bf16_kernel(const uint4* __restrict__ in,
                                                        uint4* __restrict__ out,
                                                        float* __restrict__ vscale, int role, Geom g,
                                                        const float* __restrict__ tile_amax) {
    __shared__ uint16_t tile[BS * 128];
    __shared__ uint32_t red[4];
    const long long blk = blockIdx.x;
    uint4* dst = out + blk * (BS * 16);
    constexpr int kChunks = BS * 16;
    const BlockOrigin org = block_origin(g, blockIdx.x);
    auto load = [&](int c) {                               // chunk c = 8 channels (c & 15) of slot c >> 4
        const uint4* row = token_row<RASTER>(in, g, org, blockIdx.x, c >> 4);
        return row ? row[c & 15] : make_uint4(0, 0, 0, 0);
    };
    if (role == FPS_ROLE_Q) {
        for (int c = threadIdx.x; c < kChunks; c += 256) dst[c] = load(c);
        return;
    }
    if (role == FPS_ROLE_K) {
        for (int c = threadIdx.x; c < kChunks; c += 256) {
            const int j = c >> 4, c8 = c & 15;             // row, 8-channel chunk
            if (BS == 128) {                               // 32x32x16 operand: lane 32h + n, step ks
                const int kb = j >> 5, n = j & 31, ks = c8 >> 1, h = c8 & 1;
                dst[(kb * 8 + ks) * 64 + 32 * h + n] = load(c);
            } else {
                const int b = j >> 4, n = j & 15, ks = c8 >> 2, gg = c8 & 3;
                dst[(b * 4 + ks) * 64 + gg * 16 + n] = load(c);
            }
        }
        return;
    }
    uint4* t4 = reinterpret_cast<uint4*>(tile);
    uint32_t mb = 0;
    for (int c = threadIdx.x; c < kChunks; c += 256) {
        const uint4 v = load(c);
        t4[c] = v;
        mb = amax_bits16(v, mb);
    }
    float amax;
    if (tile_amax) {
        amax = tile_amax[blk / g.KBS];
        __syncthreads();
    } else {
        mb = block_max_256(mb, red);                       // also orders the LDS writes above
        amax = __uint_as_float(mb << 16);
    }
    const int e = pow2_exponent_for_fp16(amax);
    const float down = __uint_as_float((uint32_t)(127 - e) << 23);     // 2^-e
    if (!tile_amax && threadIdx.x == 0) vscale[blk] = __uint_as_float((uint32_t)(127 + e) << 23);
    for (int c = threadIdx.x; c < kChunks; c += 256) {
        const int lane = c & 63;
        union { uint4 v; _Float16 h[8]; } o;
        if (BS == 128) {
            const int kk = (c >> 6) & 7, db = c >> 9, hh = lane >> 5, n = lane & 31;
#pragma unroll
            for (int el = 0; el < 8; ++el) {
                const int key = 32 * (kk >> 1) + 8 * (2 * (kk & 1) + (el >> 2)) + 4 * hh + (el & 3);
                const uint32_t bits = tile[key * 128 + 32 * db + n];
                o.h[el] = (_Float16)(__uint_as_float(bits << 16) * down);
            }
        } else {
            const int cb = (c >> 6) & 7, kk = c >> 9, gg = lane >> 4, n = lane & 15;
#pragma unroll
            for (int el = 0; el < 8; ++el) {
                const uint32_t bits = tile[(32 * kk + key_of_slot(gg, el)) * 128 + 16 * cb + n];
                o.h[el] = (_Float16)(__uint_as_float(bits << 16) * down);
            }
        }
        dst[c] = o.v;
    }
}

// ---- debug unpack of E4M3 tensors ---------------------------------------------------------------
template <int BS>
__global__ __launch_bounds__(256) void unpack_q8_kernel(const uint8_t* __restrict__ in,
                                                        uint8_t* __restrict__ out, int role) {
    const long long blk = blockIdx.x;
    const uint8_t* src = in + blk * (BS * 128);
    uint8_t* dst = out + blk * (BS * 128);
    for (int i = threadIdx.x; i < BS * 128; i += 256) {
        const int j = i >> 7, c = i & 127;                 // token, channel of the row-major output
        int off;
        if (role == FPS_ROLE_Q) {
            off = i;
        } else if (role == FPS_ROLE_K) {
            if (BS == 128) {
                const int kb = j >> 5, n = j & 31, ks = c >> 6, h = (c >> 5) & 1, e = (c >> 4) & 1;
                off = (((kb * 2 + ks) * 2 + e) * 64 + 32 * h + n) * 16 + (c & 15);
            } else {
                const int b = j >> 4, n = j & 15, gg = c >> 5, h = (c >> 4) & 1;
                off = ((b * 2 + h) * 64 + gg * 16 + n) * 16 + (c & 15);
            }
        } else if (BS == 128) {                            // inverse of the wide key order
            const int db = c >> 5, n = c & 31;
            const int kb = j >> 5, rem = j & 31, h = (rem >> 2) & 1, jj = 4 * (rem >> 3) + (rem & 3);
            off = (((db * 2 + (kb >> 1)) * 2 + (kb & 1)) * 64 + 32 * h + n) * 16 + jj;
        } else {
            const int cb = c >> 4, n = c & 15;
            const int gg = (j >> 2) & 3, s = 4 * (j >> 4) + (j & 3);   // inverse of key_of_slot
            off = (cb * 64 + gg * 16 + n) * 8 + s;
        }
        dst[i] = src[off];
    }
}

// ---- plain copy (calibration of HBM traffic counters against a kernel of known size) ------------
__global__ void copy_kernel(const uint4* __restrict__ in, uint4* __restrict__ out, long long n_chunks) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_chunks) out[i] = in[i];
}

static inline int grid_for(long long n, int block) { return (int)((n + block - 1) / block); }

int launch_tile_order(const Geom& g, const void* in, void* out, hipStream_t st) {
    const long long n = (long long)g.BH * g.M * g.TSP * 16;
    tile_order_kernel<<<grid_for(n, 256), 256, 0, st>>>((const uint4*)in, (uint4*)out, g, n);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? FPS_OK : hip_fail(e, "tile_order launch");
}

int launch_tile_unorder(const Geom& g, const void* in, int elem_bytes, void* out, hipStream_t st) {
    const int cpr = kHeadDim * elem_bytes / 16;
    const long long n = (long long)g.BH * g.T * g.H * g.W * cpr;
    tile_unorder_kernel<<<grid_for(n, 256), 256, 0, st>>>((const uint4*)in, (uint4*)out, g, cpr, n);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? FPS_OK : hip_fail(e, "tile_unorder launch");
}

int launch_copy(const void* in, void* out, long long bytes, hipStream_t st) {
    const long long n = bytes / 16;
    copy_kernel<<<grid_for(n, 256), 256, 0, st>>>((const uint4*)in, (uint4*)out, n);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? FPS_OK : hip_fail(e, "copy launch");
}

int launch_pack_bf16(const Geom& g, const void* x, int raster, int role, void* xp, float* vscale,
                     hipStream_t st) {
    const int blocks = g.BH * g.M * g.KB, ntiles = g.BH * g.M * g.NS;   // ntiles: quantisation groups
    const float* tile_amax = nullptr;
    if (role == FPS_ROLE_V && g.KBS > 1) {                  // `vscale` holds the tile amax meanwhile
        clear_kernel<<<(ntiles + 255) / 256, 256, 0, st>>>((uint32_t*)vscale, ntiles);
        if (raster) block_amax_kernel<true><<<blocks, 256, 0, st>>>((const uint4*)x, (uint32_t*)vscale, g);
        else        block_amax_kernel<false><<<blocks, 256, 0, st>>>((const uint4*)x, (uint32_t*)vscale, g);
        tile_amax = vscale;
    }
    const uint4* xi = (const uint4*)x;
    uint4* xo = (uint4*)xp;
    if (g.BS == 128) {
        if (raster) pack_bf16_kernel<128, true><<<blocks, 256, 0, st>>>(xi, xo, vscale, role, g, tile_amax);
        else        pack_bf16_kernel<128, false><<<blocks, 256, 0, st>>>(xi, xo, vscale, role, g, tile_amax);
    } else {
        if (raster) pack_bf16_kernel<32, true><<<blocks, 256, 0, st>>>(xi, xo, vscale, role, g, tile_amax);
        else        pack_bf16_kernel<32, false><<<blocks, 256, 0, st>>>(xi, xo, vscale, role, g, tile_amax);
    }
    if (tile_amax) amax_to_pow2_kernel<<<(ntiles + 255) / 256, 256, 0, st>>>(vscale, ntiles);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? FPS_OK : hip_fail(e, "pack_bf16 launch");
}

int launch_unpack_q8(const Geom& g, const void* xq, int role, uint8_t* out, hipStream_t st) {
    const int blocks = g.BH * g.M * g.KB;
    if (g.BS == 128) unpack_q8_kernel<128><<<blocks, 256, 0, st>>>((const uint8_t*)xq, out, role);
    else             unpack_q8_kernel<32><<<blocks, 256, 0, st>>>((const uint8_t*)xq, out, role);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? FPS_OK : hip_fail(e, "unpack_q8 launch");
}

}  // namespace fps
