// Sliding-tile attention forward (Eq. 2-3, Sec. 3.2 aggregation; Algorithm 1 steps 4-5).
//
// One workgroup per (bh, query tile); wave w owns query rows 32w..32w+31 of the tile as two
// 16-row blocks.  The kernel walks the box of key tiles given by Eq. 2 -- tile pairs outside the
// box are never scheduled -- staging each K and V tile through LDS.  Scores are produced
// transposed, S^T = K Q^T, so that a lane's accumulator holds one query row and the keys
// 16b + 4g + 0..3; after the softmax those registers are, unchanged, the second operand of the
// PV product O^T = V^T P^T (see the packed layouts in fps_layout.hip).
//
// Softmax is online in base 2 with an integer row reference m (ceil of the running row maximum):
// P = 2^(S' - m) <= 1, rescaling by 2^(m_old - m_new) is exact, and the E4M3 rounding of 448*P
// does not depend on the order in which key tiles arrive (apart from values in the subnormal
// range of the format).  The denominator accumulates the unrounded P.
#include "fps_internal.h"

namespace fps {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 v2h __attribute__((ext_vector_type(2)));

struct AttnArgs {
    const uint8_t* q;
    const uint8_t* k;
    const uint8_t* v;
    const float* sq;
    const float* sk;
    const float* sv;
    void* out;
    uint8_t* visited;
    Geom g;
    int rt, rh, rw;        // window radii in tiles
    int out_f32;
    int chunk;             // work items per XCD
    int total;             // BH * M
    uint32_t partial_cls;  // bit c set iff boundary class c has padded tokens
};

constexpr float kLog2eOverSqrtD = 0.12751743f;   // log2(e) / sqrt(128)
constexpr float kLog2Of448 = 8.8073549f;          // log2(448)

// Scales are read-only for the whole launch and indexed uniformly: reading them through the constant
// address space lets the compiler use scalar loads, which do not queue behind the vector-memory
// traffic that stages the K/V tiles.
typedef const __attribute__((address_space(4))) float* const_f32_ptr;
__device__ __forceinline__ float load_uniform(const float* p, size_t i) {
    return ((const_f32_ptr)(uintptr_t)p)[i];
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
    const uint32_t u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// Work item of this workgroup.  Workgroups are dealt round-robin to the 8 XCDs by the hardware;
// giving XCD x the contiguous range [x*chunk, (x+1)*chunk) of (bh, tile) items keeps the key
// tiles of neighbouring query tiles of one head in that XCD's L2.
__device__ __forceinline__ bool work_item(const AttnArgs& a, int* bh, int* u) {
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int wi = xcd * a.chunk + slot;
    if (slot >= a.chunk || wi >= a.total) return false;
    *bh = wi / a.g.M;
    *u = wi - *bh * a.g.M;
    return true;
}

__device__ __forceinline__ int tile_class(const Geom& g, int t, int h, int w) {
    return ((t == g.nT - 1) << 2) | ((h == g.nH - 1) << 1) | (w == g.nW - 1);
}

// Epilogue shared by both precisions: O = acc * inv_l, padded rows zero, fp32 or bf16 store.
template <int TS>
__device__ __forceinline__ void store_rows(const AttnArgs& a, int bh, int u, int ucls, int wave,
                                           int g, int n, const v4f (&acc)[2][8], const float (&inv)[2]) {
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const int rr = wave * 32 + qb * 16 + n;
        const bool valid = (a.g.valid_mask[ucls][rr >> 5] >> (rr & 31)) & 1u;
        const float sc = valid ? inv[qb] : 0.0f;
        const size_t row = ((size_t)bh * a.g.M + u) * TS + rr;
#pragma unroll
        for (int cb = 0; cb < 8; ++cb) {
            v4f o = acc[qb][cb] * sc;
            if (!valid) o = v4f{0.f, 0.f, 0.f, 0.f};
            const int col = 16 * cb + 4 * g;
            if (a.out_f32) {
                *reinterpret_cast<v4f*>(reinterpret_cast<float*>(a.out) + row * 128 + col) = o;
            } else {
                uint2 pk;
                pk.x = f32_to_bf16_bits(o[0]) | (f32_to_bf16_bits(o[1]) << 16);
                pk.y = f32_to_bf16_bits(o[2]) | (f32_to_bf16_bits(o[3]) << 16);
                *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(a.out) + row * 128 + col) = pk;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// FP8 E4M3: both products on v_mfma_f32_16x16x128_f8f6f4 (TS = 128) or, for the PV product of
// 32-token tiles, v_mfma_f32_16x16x32_fp8_fp8.
// ---------------------------------------------------------------------------------------------
// Walks the key-tile box of Eq. 2 in (t, h, w) order.
struct TileWalk {
    int t0, h0, w0, h1, w1;
    int vt, vh, vw;
    int n;                                  // number of tiles in the box
    __device__ __forceinline__ void init(const AttnArgs& a, int ut, int uh, int uw) {
        const Geom& G = a.g;
        t0 = max(0, ut - a.rt); h0 = max(0, uh - a.rh); w0 = max(0, uw - a.rw);
        const int t1 = min(G.nT - 1, ut + a.rt);
        h1 = min(G.nH - 1, uh + a.rh); w1 = min(G.nW - 1, uw + a.rw);
        n = (t1 - t0 + 1) * (h1 - h0 + 1) * (w1 - w0 + 1);
        vt = t0; vh = h0; vw = w0;
    }
    __device__ __forceinline__ void next() {
        if (++vw > w1) { vw = w0; if (++vh > h1) { vh = h0; ++vt; } }
    }
};

// State of one wave of attn_fp8_kernel: two 16-row query blocks, their softmax statistics and
// output accumulators.
template <int TS>
struct Fp8Wave {
    static constexpr int NB = TS / 16;
    v8i qop[2];
    float m_run[2];
    float l_run[2];          // running sum of 448 * P
    v4f acc[2][8];
};

__device__ __forceinline__ v8i make_v8i(const uint4& lo, const uint4& hi) {
    return v8i{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
}

// One key tile: S^T = K Q^T, masked online softmax, P quantised to E4M3, O^T += s^V (V^T P^T).
// ldsK / ldsV are the staged operand tiles (packed layouts of fps_layout.hip).
template <int TS>
__device__ __forceinline__ void fp8_tile(Fp8Wave<TS>& w, const AttnArgs& a, const uint8_t* ldsK,
                                         const uint8_t* ldsV, int lane, int g, float sc, float svv,
                                         int cls) {
    constexpr int NB = TS / 16;
    const Geom& G = a.g;
    const uint4* ldsK4 = reinterpret_cast<const uint4*>(ldsK);
    const uint4* ldsV4 = reinterpret_cast<const uint4*>(ldsV);

    // K operands are fetched two blocks ahead of the MFMA that consumes them
    v4f s[2][NB];
    uint4 klo[2], khi[2];
    klo[0] = ldsK4[0 * 64 + lane]; khi[0] = ldsK4[1 * 64 + lane];
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        if (b + 1 < NB) {
            klo[(b + 1) & 1] = ldsK4[((b + 1) * 2 + 0) * 64 + lane];
            khi[(b + 1) & 1] = ldsK4[((b + 1) * 2 + 1) * 64 + lane];
        }
        const v8i kop = make_v8i(klo[b & 1], khi[b & 1]);
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
            s[qb][b] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(
                kop, w.qop[qb], v4f{0.f, 0.f, 0.f, 0.f}, 0, 0, 0, 0, 0, 0);
    }
    // first V operands are requested now so that they arrive during the softmax
    uint4 vlo[2], vhi[2];
    long v32[2];
    if constexpr (TS == 128) {
        vlo[0] = ldsV4[0 * 64 + lane]; vhi[0] = ldsV4[1 * 64 + lane];
    } else {
        v32[0] = reinterpret_cast<const long*>(ldsV)[0 * 64 + lane];
    }

    if ((a.partial_cls >> cls) & 1u) {                     // padded keys of a boundary tile: -inf
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const uint32_t bits = G.valid_mask[cls][b >> 1] >> (((b & 1) << 4) + 4 * g);
#pragma unroll
            for (int r = 0; r < 4; ++r)
                if (!((bits >> r) & 1u)) { s[0][b][r] = -INFINITY; s[1][b][r] = -INFINITY; }
        }
    }

    int pb[2][NB];                                         // P^T as packed E4M3, 4 keys per dword
    float alpha[2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        float mx = __builtin_fmaxf(__builtin_fmaxf(s[qb][0][0], s[qb][0][1]),
                                   __builtin_fmaxf(s[qb][0][2], s[qb][0][3]));
#pragma unroll
        for (int b = 1; b < NB; ++b) {
            mx = __builtin_fmaxf(__builtin_fmaxf(mx, s[qb][b][0]), s[qb][b][1]);
            mx = __builtin_fmaxf(__builtin_fmaxf(mx, s[qb][b][2]), s[qb][b][3]);
        }
        mx = __builtin_fmaxf(mx, __shfl_xor(mx, 16));
        mx = __builtin_fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = __builtin_fmaxf(w.m_run[qb], __builtin_ceilf(mx * sc));
        alpha[qb] = fast_exp2(w.m_run[qb] - m_new);
        w.m_run[qb] = m_new;
        // 448 * 2^(S' - m) = 2^(S' + (log2(448) - m)): the factor 448 rides in the exponent
        const float cm = kLog2Of448 - m_new;
        float rs = 0.f;
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            float p[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                p[r] = fast_exp2(__builtin_fmaf(s[qb][b][r], sc, cm));
                rs += p[r];
            }
            int pw = 0;
            pw = __builtin_amdgcn_cvt_pk_fp8_f32(p[0], p[1], pw, false);
            pw = __builtin_amdgcn_cvt_pk_fp8_f32(p[2], p[3], pw, true);
            pb[qb][b] = pw;
        }
        w.l_run[qb] = w.l_run[qb] * alpha[qb] + rs;
    }
    // the row reference rarely moves after the first tiles: rescale O only when some row needs it
    if (__any(alpha[0] != 1.0f || alpha[1] != 1.0f)) {
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int cb = 0; cb < 8; ++cb) w.acc[qb][cb] *= alpha[qb];
    }

    // O^T += s^V_v * (V^T P^T)
#pragma unroll
    for (int cb = 0; cb < 8; ++cb) {
        if constexpr (TS == 128) {
            if (cb + 1 < 8) {
                vlo[(cb + 1) & 1] = ldsV4[((cb + 1) * 2 + 0) * 64 + lane];
                vhi[(cb + 1) & 1] = ldsV4[((cb + 1) * 2 + 1) * 64 + lane];
            }
            const v8i vop = make_v8i(vlo[cb & 1], vhi[cb & 1]);
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                const v8i pop = v8i{pb[qb][0], pb[qb][1], pb[qb][2], pb[qb][3],
                                    pb[qb][4], pb[qb][5], pb[qb][6], pb[qb][7]};
                const v4f t = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(
                    vop, pop, v4f{0.f, 0.f, 0.f, 0.f}, 0, 0, 0, 0, 0, 0);
                w.acc[qb][cb] += t * svv;
            }
        } else {
            if (cb + 1 < 8) v32[(cb + 1) & 1] = reinterpret_cast<const long*>(ldsV)[(cb + 1) * 64 + lane];
            const long vop = v32[cb & 1];
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                const long pop = (long)(uint32_t)pb[qb][0] | ((long)(uint32_t)pb[qb][1] << 32);
                const v4f t = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(
                    vop, pop, v4f{0.f, 0.f, 0.f, 0.f}, 0, 0, 0);
                w.acc[qb][cb] += t * svv;
            }
        }
    }
}

template <int TS>
__global__ __launch_bounds__(TS * 2) __attribute__((amdgpu_waves_per_eu(2, 2)))
void attn_fp8_kernel(AttnArgs a) {
    constexpr int NTHR = TS * 2;
    constexpr int CPT = (TS * 8) / NTHR;                   // 16-byte chunks per thread per operand tile
    constexpr int TILE_BYTES = TS * 128;
    // Two staging buffers, each (K tile, V tile), as separate objects: the next tile streams into
    // one while the other is read, and the compiler can tell the two apart.
    __shared__ __attribute__((aligned(16))) uint8_t ldsA[2][TILE_BYTES];
    __shared__ __attribute__((aligned(16))) uint8_t ldsB[2][TILE_BYTES];
    int bh, u;
    if (!work_item(a, &bh, &u)) return;
    const Geom& G = a.g;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 4, n = lane & 15;
    const int uw = u % G.nW, uh = (u / G.nW) % G.nH, ut = u / (G.nW * G.nH);
    const size_t tile0 = (size_t)bh * G.M;

    Fp8Wave<TS> w;
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const int row = wave * 32 + qb * 16 + n;
        const uint4* p = reinterpret_cast<const uint4*>(a.q + ((tile0 + u) * TS + row) * 128 + 32 * g);
        w.qop[qb] = make_v8i(p[0], p[1]);
        w.m_run[qb] = -INFINITY;
        w.l_run[qb] = 0.f;
#pragma unroll
        for (int cb = 0; cb < 8; ++cb) w.acc[qb][cb] = v4f{0.f, 0.f, 0.f, 0.f};
    }
    const float sqc = load_uniform(a.sq, tile0 + u) * kLog2eOverSqrtD;

    TileWalk walk;
    walk.init(a, ut, uh, uw);

    // HBM -> LDS staging is a linear copy done by the load unit itself (global_load_lds_dwordx4:
    // lane i of a wave deposits its 16 bytes at the wave's LDS base + 16 i), so no VGPRs are spent
    auto stage = [&](uint8_t (*dst)[TILE_BYTES], int v) {
        const uint4* gk = reinterpret_cast<const uint4*>(a.k + (tile0 + v) * TILE_BYTES);
        const uint4* gv = reinterpret_cast<const uint4*>(a.v + (tile0 + v) * TILE_BYTES);
#pragma unroll
        for (int c = 0; c < CPT; ++c) {
            const int chunk0 = c * NTHR + wave * 64;       // wave-uniform
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void*)(gk + chunk0 + lane),
                (__attribute__((address_space(3))) void*)(&dst[0][chunk0 * 16]), 16, 0, 0);
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void*)(gv + chunk0 + lane),
                (__attribute__((address_space(3))) void*)(&dst[1][chunk0 * 16]), 16, 0, 0);
        }
    };
    auto tile_id = [&]() { return (walk.vt * G.nH + walk.vh) * G.nW + walk.vw; };

    stage(ldsA, tile_id());
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    // one key tile per half-iteration: compute from `cur` while the next tile lands in `nxt`
    auto half = [&](uint8_t (*cur)[TILE_BYTES], uint8_t (*nxt)[TILE_BYTES], int it) {
        const int v = tile_id();
        const int cls = tile_class(G, walk.vt, walk.vh, walk.vw);
        const float sc = sqc * load_uniform(a.sk, tile0 + v);
        const float svv = load_uniform(a.sv, tile0 + v);
        if (a.visited && bh == 0 && tid == 0) a.visited[(size_t)u * G.M + v] = 1;
        walk.next();
        if (it + 1 < walk.n) stage(nxt, tile_id());
        fp8_tile<TS>(w, a, cur[0], cur[1], lane, g, sc, svv, cls);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this thread's share of the next tile landed
        __syncthreads();
    };
    for (int it = 0; it < walk.n; it += 2) {
        half(ldsA, ldsB, it);
        if (it + 1 < walk.n) half(ldsB, ldsA, it + 1);
    }

    float inv[2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        float l = w.l_run[qb];
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        inv[qb] = l > 0.f ? 1.0f / l : 0.f;               // l already carries the factor 448
    }
    store_rows<TS>(a, bh, u, tile_class(G, ut, uh, uw), wave, g, n, w.acc, inv);
}

// ---------------------------------------------------------------------------------------------
// BF16: no quantisation.  K Q^T on v_mfma_f32_16x16x32_bf16; P is rounded to fp16 and multiplied
// with the fp16 V tiles (exact per-tile power-of-two scaling, undone by s^V) on
// v_mfma_f32_16x16x32_f16.
// ---------------------------------------------------------------------------------------------
union Bf16x8 { uint4 u; v8bf v; v8h h; };

template <int TS>
__global__ __launch_bounds__(TS * 2) void attn_bf16_kernel(AttnArgs a) {
    constexpr int NB = TS / 16;
    constexpr int NKK = TS / 32;
    constexpr int NTHR = TS * 2;
    __shared__ __attribute__((aligned(16))) uint8_t ldsK[TS * 256];
    __shared__ __attribute__((aligned(16))) uint8_t ldsV[TS * 256];
    int bh, u;
    if (!work_item(a, &bh, &u)) return;
    const Geom& G = a.g;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 4, n = lane & 15;
    const int uw = u % G.nW, uh = (u / G.nW) % G.nH, ut = u / (G.nW * G.nH);
    const size_t tile0 = (size_t)bh * G.M;

    Bf16x8 qop[2][4];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const int row = wave * 32 + qb * 16 + n;
        const uint4* p = reinterpret_cast<const uint4*>(a.q + ((tile0 + u) * TS + row) * 256);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) qop[qb][ks].u = p[ks * 4 + g];
    }

    float m_run[2] = {-INFINITY, -INFINITY};
    float l_run[2] = {0.f, 0.f};
    v4f acc[2][8];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int cb = 0; cb < 8; ++cb) acc[qb][cb] = v4f{0.f, 0.f, 0.f, 0.f};

    const int t0 = max(0, ut - a.rt), t1 = min(G.nT - 1, ut + a.rt);
    const int h0 = max(0, uh - a.rh), h1 = min(G.nH - 1, uh + a.rh);
    const int w0 = max(0, uw - a.rw), w1 = min(G.nW - 1, uw + a.rw);
    const uint4* ldsK4 = reinterpret_cast<const uint4*>(ldsK);
    const uint4* ldsV4 = reinterpret_cast<const uint4*>(ldsV);
    const float sc = kLog2eOverSqrtD;

    for (int vt = t0; vt <= t1; ++vt)
    for (int vh = h0; vh <= h1; ++vh)
    for (int vw = w0; vw <= w1; ++vw) {
        const int v = (vt * G.nH + vh) * G.nW + vw;
        __syncthreads();
        {
            const uint4* gk = reinterpret_cast<const uint4*>(a.k + (tile0 + v) * TS * 256);
            const uint4* gv = reinterpret_cast<const uint4*>(a.v + (tile0 + v) * TS * 256);
            for (int c = tid; c < TS * 16; c += NTHR) {
                reinterpret_cast<uint4*>(ldsK)[c] = gk[c];
                reinterpret_cast<uint4*>(ldsV)[c] = gv[c];
            }
        }
        __syncthreads();
        const int cls = tile_class(G, vt, vh, vw);
        const float svv = a.sv[tile0 + v];
        if (a.visited && bh == 0 && tid == 0) a.visited[(size_t)u * G.M + v] = 1;

        v4f s[2][NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            s[0][b] = v4f{0.f, 0.f, 0.f, 0.f};
            s[1][b] = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                Bf16x8 kop;
                kop.u = ldsK4[(b * 4 + ks) * 64 + lane];
#pragma unroll
                for (int qb = 0; qb < 2; ++qb)
                    s[qb][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kop.v, qop[qb][ks].v, s[qb][b], 0, 0, 0);
            }
        }
        if ((a.partial_cls >> cls) & 1u) {
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const uint32_t bits = G.valid_mask[cls][b >> 1] >> (((b & 1) << 4) + 4 * g);
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (!((bits >> r) & 1u)) { s[0][b][r] = -INFINITY; s[1][b][r] = -INFINITY; }
            }
        }

        Bf16x8 pop[2][NKK];
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            float mx = s[qb][0][0];
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int r = 0; r < 4; ++r) mx = __builtin_fmaxf(mx, s[qb][b][r]);
            mx = __builtin_fmaxf(mx, __shfl_xor(mx, 16));
            mx = __builtin_fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new = __builtin_fmaxf(m_run[qb], __builtin_ceilf(mx * sc));
            const float alpha = fast_exp2(m_run[qb] - m_new);
            m_run[qb] = m_new;
            float rs = 0.f;
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                float p[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    p[r] = fast_exp2(__builtin_fmaf(s[qb][b][r], sc, -m_new));
                    rs += p[r];
                }
#pragma unroll
                for (int r = 0; r < 4; ++r) pop[qb][b >> 1].h[(b & 1) * 4 + r] = (_Float16)p[r];
            }
            l_run[qb] = l_run[qb] * alpha + rs;
#pragma unroll
            for (int cb = 0; cb < 8; ++cb) acc[qb][cb] *= alpha;
        }

#pragma unroll
        for (int cb = 0; cb < 8; ++cb) {
            v4f t[2] = {v4f{0.f, 0.f, 0.f, 0.f}, v4f{0.f, 0.f, 0.f, 0.f}};
#pragma unroll
            for (int kk = 0; kk < NKK; ++kk) {
                Bf16x8 vop;
                vop.u = ldsV4[(kk * 8 + cb) * 64 + lane];
#pragma unroll
                for (int qb = 0; qb < 2; ++qb)
                    t[qb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(vop.h, pop[qb][kk].h, t[qb], 0, 0, 0);
            }
            acc[0][cb] += t[0] * svv;
            acc[1][cb] += t[1] * svv;
        }
    }

    float inv[2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        float l = l_run[qb];
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        inv[qb] = l > 0.f ? 1.0f / l : 0.f;
    }
    store_rows<TS>(a, bh, u, tile_class(G, ut, uh, uw), wave, g, n, acc, inv);
}

// Debug: raw E4M3 score accumulators sum_c q_ic * k_jc of one tile pair, produced by the same MFMA
// instruction and operand layouts as attn_fp8_kernel; out[i*TS + j], query-major.
template <int TS>
__global__ __launch_bounds__(TS * 2) void scores_fp8_kernel(const uint8_t* __restrict__ q,
                                                            const uint8_t* __restrict__ k,
                                                            float* __restrict__ out) {
    constexpr int NB = TS / 16;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 4, n = lane & 15;
    const uint4* k4 = reinterpret_cast<const uint4*>(k);
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const int row = wave * 32 + qb * 16 + n;
        const uint4* p = reinterpret_cast<const uint4*>(q + row * 128 + 32 * g);
        const uint4 lo = p[0], hi = p[1];
        const v8i qop = v8i{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
        for (int b = 0; b < NB; ++b) {
            const uint4 klo = k4[(b * 2 + 0) * 64 + lane], khi = k4[(b * 2 + 1) * 64 + lane];
            const v8i kop = v8i{(int)klo.x, (int)klo.y, (int)klo.z, (int)klo.w, (int)khi.x, (int)khi.y, (int)khi.z, (int)khi.w};
            const v4f s = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(
                kop, qop, v4f{0.f, 0.f, 0.f, 0.f}, 0, 0, 0, 0, 0, 0);
#pragma unroll
            for (int r = 0; r < 4; ++r) out[row * TS + 16 * b + 4 * g + r] = s[r];
        }
    }
}

int launch_scores_fp8(const Geom& g, const void* q, const void* k, int bh, int u, int v, float* out,
                      hipStream_t st) {
    const size_t tile_bytes = (size_t)g.TS * 128;
    const uint8_t* qp = (const uint8_t*)q + ((size_t)bh * g.M + u) * tile_bytes;
    const uint8_t* kp = (const uint8_t*)k + ((size_t)bh * g.M + v) * tile_bytes;
    if (g.TS == 128) scores_fp8_kernel<128><<<1, 256, 0, st>>>(qp, kp, out);
    else             scores_fp8_kernel<32><<<1, 64, 0, st>>>(qp, kp, out);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? FPS_OK : hip_fail(e, "debug scores launch");
}

int launch_attn(const Geom& g, const fps_window& win, int prec, const void* q, const void* k,
                const void* v, const float* sq, const float* sk, const float* sv, int vscale,
                void* out, int out_f32, uint8_t* visited, hipStream_t st) {
    if (prec == FPS_PREC_FP8 && vscale != FPS_VSCALE_TILE) {
        set_error("per-channel V scales are not implemented yet");
        return FPS_ERR_UNSUPPORTED;
    }
    AttnArgs a;
    a.q = (const uint8_t*)q; a.k = (const uint8_t*)k; a.v = (const uint8_t*)v;
    a.sq = sq; a.sk = sk; a.sv = sv;
    a.out = out; a.visited = visited;
    a.g = g;
    a.rt = win.wt / 2; a.rh = win.wh / 2; a.rw = win.ww / 2;
    a.out_f32 = out_f32;
    a.total = g.BH * g.M;
    a.chunk = (a.total + 7) / 8;
    a.partial_cls = 0;
    const int full_words = g.TS / 32;
    for (int c = 0; c < 8; ++c)
        for (int w = 0; w < full_words; ++w)
            if (g.valid_mask[c][w] != 0xFFFFFFFFu) a.partial_cls |= 1u << c;
    const int grid = a.chunk * 8;
    if (prec == FPS_PREC_FP8) {
        if (g.TS == 128) attn_fp8_kernel<128><<<grid, 256, 0, st>>>(a);
        else             attn_fp8_kernel<32><<<grid, 64, 0, st>>>(a);
    } else {
        if (g.TS == 128) attn_bf16_kernel<128><<<grid, 256, 0, st>>>(a);
        else             attn_bf16_kernel<32><<<grid, 64, 0, st>>>(a);
    }
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? FPS_OK : hip_fail(e, "attention launch");
}

}  // namespace fps
