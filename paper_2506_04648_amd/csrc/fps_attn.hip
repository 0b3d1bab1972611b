// Sliding-tile attention forward (Eq. 2-3, Sec. 3.2 aggregation; Algorithm 1 steps 4-5).
//
// One workgroup per (bh, query tile, block of BS = 128 or 32 query slots of the tile).  The kernel
// walks the box of key tiles given by Eq. 2 -- tile pairs outside the box are never scheduled --
// block by block, staging each K and V block through LDS.  A tile of at most BS tokens is one
// block; larger tiles, and tiles cut into quantisation sub-tiles, are several blocks (kernels
// instantiated with MB = true).  Scores are produced transposed, S^T = K Q^T, so that a lane's
// accumulator holds one query row and a fixed set of keys; after the softmax those registers are,
// unchanged, the second operand of the PV product O^T = V^T P^T (see the packed layouts in
// fps_layout.hip).
//
// Four kernels share that plan.  128-slot blocks (any scale group of more than 96 tokens) run on
// the 32x32 matrix instructions: attn_fp8_wide_kernel, attn_bf16_wide_kernel; a wave of 64 lanes owns
// 32 query rows.  32-slot blocks (small tiles) run on the 16x16 instructions: attn_fp8_kernel<32>,
// attn_bf16_kernel<32>; the single wave owns 32 query rows as two 16-row blocks.  The 16x16 kernels
// are written for either block size but only instantiated for 32.
//
// Softmax is online in base 2 with an integer row reference m (ceil of the running row maximum):
// P = 2^(S' - m) <= 1, rescaling by 2^(m_old - m_new) is exact, and the E4M3 rounding of 448*P
// does not depend on the order in which key tiles arrive (apart from values in the subnormal
// range of the format).  The denominator accumulates the unrounded P.
#include "fps_internal.h"

#include <cstddef>
#include <cstring>
#include <type_traits>

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
    int edge_shift;        // 1: clamp the window centre into the grid instead of truncating
    int out_f32;
    int out_raster;        // output in raster order (real tokens only) instead of tile order
    int chunk;             // work items per XCD
    int total;             // BH * M * KB
    uint32_t partial_cls;  // bit c set iff a tile of boundary class c has padding slots
};

// Second kernel parameter, used by the one-block-per-tile kernels only.  They never name it: they
// read it through the kernel-argument segment pointer (constant address space), so a wave-uniform
// index gives scalar loads and the table is never copied to private memory.
struct MaskTables {
    // lane_mask[c][4b + r]: bit of lane (n, g) set iff the key that lane holds in accumulator slot
    // (block b, element r), slot 16b + 4g + r of a one-block tile, is a real token (class c)
    uint64_t lane_mask[8][32];
    // 128-slot blocks (32x32 accumulators): see arg_pair_code
    uint32_t pair_code[8][4];
};
constexpr size_t kTablesOffset = (sizeof(AttnArgs) + 7) & ~size_t(7);   // kernarg offset of MaskTables

// Every lambda of the kernels captures the accumulators by reference; left to the inliner's cost
// model a large one stays a call, which forces everything it captures into private memory.
#define FPS_INLINE __attribute__((always_inline))

constexpr float kLog2eOverSqrtD = 0.12751743f;   // log2(e) / sqrt(128)
constexpr float kLog2Of448 = 8.8073549f;          // log2(448)
constexpr float kFp16PScaleLog2 = 14.0f;          // BF16 mode holds 2^14 * P in fp16
constexpr float kMaxDrift = 64.0f;                // largest m - m_base before O and l are moved to a new reference
constexpr int kStoreRegionBytes = 16 * (512 + 16);  // per-wave LDS region of the output transpose

// Scales are read-only for the whole launch and indexed uniformly: reading them through the constant
// address space lets the compiler use scalar loads, which do not queue behind the vector-memory
// traffic that stages the K/V tiles.
typedef const __attribute__((address_space(4))) float* const_f32_ptr;
__device__ __forceinline__ float load_uniform(const float* p, size_t i) {
    return ((const_f32_ptr)(uintptr_t)p)[i];
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Reductions over the four lanes n, n+16, n+32, n+48 that hold one query row.  gfx950 swaps rows of
// 16 lanes (and halves of 32) between two registers at VALU speed: with both operands equal to t,
// v_permlane16_swap leaves (r0,r0,r2,r2) and (r1,r1,r3,r3), v_permlane32_swap (lo,lo) and (hi,hi),
// so two swaps and two combines replace two LDS-routed shuffles and their latency.
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float max_over_row_lanes(float t) {
    u32x2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(t), __float_as_uint(t), false, false);
    t = __builtin_fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
    r = __builtin_amdgcn_permlane32_swap(__float_as_uint(t), __float_as_uint(t), false, false);
    return __builtin_fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_over_row_lanes(float t) {
    u32x2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(t), __float_as_uint(t), false, false);
    t = __uint_as_float(r[0]) + __uint_as_float(r[1]);
    r = __builtin_amdgcn_permlane32_swap(__float_as_uint(t), __float_as_uint(t), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// two floats -> two bf16 (round to nearest even) in one dword; gfx950 converts in hardware
typedef float v2f __attribute__((ext_vector_type(2)));
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v2f{lo, hi}, v2bf));
}

// Work item of this workgroup.  Workgroups are dealt round-robin to the 8 XCDs by the hardware;
// giving XCD x the contiguous range [x*chunk, (x+1)*chunk) of (bh, tile) items keeps the key
// tiles of neighbouring query tiles of one head in that XCD's L2.
// A work item is one block of BS query rows: (bh, query tile u, block jq of the tile).
__device__ __forceinline__ bool work_item(const AttnArgs& a, int KB, int* bh, int* u, int* jq) {
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int wi = xcd * a.chunk + slot;
    if (slot >= a.chunk || wi >= a.total) return false;
    const int tile_lin = wi / KB;
    *jq = wi - tile_lin * KB;
    *bh = tile_lin / a.g.M;
    *u = tile_lin - *bh * a.g.M;
    return true;
}

// Tables inside the kernel-argument block, read through the constant address space with a
// wave-uniform index so that they come in by scalar loads (indexing the by-value argument struct
// directly can make the compiler spill it to private memory).
__device__ __forceinline__ uint64_t arg_lane_mask(int cls, int i) {
    typedef const __attribute__((address_space(4))) uint64_t* ptr_t;
    const __attribute__((address_space(4))) char* base =
        (const __attribute__((address_space(4))) char*)__builtin_amdgcn_kernarg_segment_ptr();
    return ((ptr_t)(base + kTablesOffset + offsetof(MaskTables, lane_mask)))[cls * 32 + i];
}
// x where the lane's bit of the wave-uniform mask is set, otherwise y: one v_cndmask with the mask
// taken straight from scalar registers (no per-lane bit extraction).
__device__ __forceinline__ float select_lanes(uint64_t lane_mask, float x, float y) {
    float out;
    asm("v_cndmask_b32_e64 %0, %1, %2, %3" : "=v"(out) : "v"(y), "v"(x), "s"(lane_mask));
    return out;
}

template <typename G_>
__device__ __forceinline__ int tile_class(const G_& g, int t, int h, int w) {
    return ((t == g.nT - 1) << 2) | ((h == g.nH - 1) << 1) | (w == g.nW - 1);
}

// Epilogue shared by both precisions: O = acc * inv_l (times the per-channel V scale if any),
// padded rows zero, fp32 or bf16, tile or raster order.  A lane holds 4 channels of one row per
// accumulator, so direct stores would be 8- or 16-byte pieces of many rows; instead each wave
// transposes its 16-row blocks through a private 16 KB LDS region and writes whole rows
// (256 or 512 contiguous bytes).  The caller guarantees that no wave still reads the LDS buffers.
template <int BS>
__device__ __forceinline__ void store_rows(const AttnArgs& a, int bh, int u, int jq, int KBS, int ucls, int wave,
                                           int lane, const v4f (&acc)[2][8], const float (&inv)[2],
                                           uint8_t* wave_lds, const float* ch_scale = nullptr) {
    const auto& G = a.g;
    const int g = lane >> 4, n = lane & 15;
    const int row_bytes = a.out_f32 ? 512 : 256;
    const int pitch = row_bytes + 16;                      // padding keeps the column writes off one bank
    const int uw = u % G.nW, uh = (u / G.nW) % G.nH, ut = u / (G.nW * G.nH);
    // the block lies in ONE sub-tile: decode that once, the rows then cost two divisions each
    const int sub = jq / KBS;
    const SubTile so = sub_tile_origin(G, sub);
    const int slot0 = (jq - sub * KBS) * BS;               // the block's first slot within the sub-tile
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
#pragma unroll
        for (int cb = 0; cb < 8; ++cb) {
            const int col = 16 * cb + 4 * g;
            v4f o = acc[qb][cb] * inv[qb];
            if (ch_scale) o *= *reinterpret_cast<const v4f*>(ch_scale + col);
            if (a.out_f32) {
                *reinterpret_cast<v4f*>(wave_lds + n * pitch + col * 4) = o;
            } else {
                uint2 pk;
                pk.x = pack_bf16x2(o[0], o[1]);
                pk.y = pack_bf16x2(o[2], o[3]);
                *reinterpret_cast<uint2*>(wave_lds + n * pitch + col * 2) = pk;
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        // whole rows: 16 lanes (bf16) or 32 lanes (fp32) per row, 16 bytes per lane
        const int lanes_shift = a.out_f32 ? 5 : 4;
        const int rows_per_pass = 64 >> lanes_shift;
        for (int r0 = 0; r0 < 16; r0 += rows_per_pass) {
            const int r = r0 + (lane >> lanes_shift), chunk = lane & ((1 << lanes_shift) - 1);
            const int in_block = wave * 32 + qb * 16 + r;       // BS: block size
            int rt = 0, rh = 0, rw = 0;
            const bool valid = sub_slot_coords(G, so, slot0 + in_block, &rt, &rh, &rw) &&
                               coords_in_class(G, ucls, rt, rh, rw);
            uint4 val = *reinterpret_cast<const uint4*>(wave_lds + r * pitch + chunk * 16);
            size_t row;
            if (a.out_raster) {
                if (!valid) continue;
                row = (((size_t)bh * G.T + (ut * G.Tt + rt)) * G.H + (uh * G.Th + rh)) * G.W + (uw * G.Tw + rw);
            } else {
                row = ((size_t)bh * G.M + u) * G.TSP + (size_t)jq * BS + in_block;
                if (!valid) val = make_uint4(0, 0, 0, 0);
            }
            reinterpret_cast<uint4*>(reinterpret_cast<uint8_t*>(a.out) + row * row_bytes)[chunk] = val;
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        __builtin_amdgcn_wave_barrier();                   // the region is reused by the next block
    }
}

// Walks the key-tile box of Eq. 2 in (t, h, w) order, block by block inside each tile.  Blocks of
// a last-along-T tile beyond kb_last hold padding only and are skipped.
struct TileWalk {
    int t0, h0, w0, h1, w1;
    int vt, vh, vw;
    int jk, kb_cur;                         // block within the tile, blocks to visit in this tile
    int js, jb, kbs;                        // jk = js * kbs + jb: sub-tile (scale group) and block in it
    int kb_full, kb_last, last_t;
    int n;                                  // number of key BLOCKS in the box
    __device__ __forceinline__ void init(const AttnArgs& a, int KB, int KB_LAST, int KBS, int ut, int uh, int uw) {
        const Geom& G = a.g;
        if (a.edge_shift) {                 // clamp the centre into [r, n-1-r]; an axis not longer than
            // the window has no such centre and is kept whole by the truncation below with u = n/2
            ut = G.nT > 2 * a.rt + 1 ? min(max(ut, a.rt), G.nT - 1 - a.rt) : G.nT / 2;
            uh = G.nH > 2 * a.rh + 1 ? min(max(uh, a.rh), G.nH - 1 - a.rh) : G.nH / 2;
            uw = G.nW > 2 * a.rw + 1 ? min(max(uw, a.rw), G.nW - 1 - a.rw) : G.nW / 2;
        }
        t0 = max(0, ut - a.rt); h0 = max(0, uh - a.rh); w0 = max(0, uw - a.rw);
        const int t1 = min(G.nT - 1, ut + a.rt);
        h1 = min(G.nH - 1, uh + a.rh); w1 = min(G.nW - 1, uw + a.rw);
        kb_full = KB; kb_last = KB_LAST; last_t = G.nT - 1;
        const int has_last = t1 == last_t;
        n = (h1 - h0 + 1) * (w1 - w0 + 1) * ((t1 - t0 + 1 - has_last) * KB + has_last * KB_LAST);
        vt = t0; vh = h0; vw = w0; jk = 0; js = 0; jb = 0; kbs = KBS;
        kb_cur = vt == last_t ? kb_last : kb_full;
    }
    __device__ __forceinline__ void next() {
        if (++jb == kbs) { jb = 0; ++js; }
        if (++jk < kb_cur) return;
        jk = 0; js = 0; jb = 0;
        if (++vw > w1) {
            vw = w0;
            if (++vh > h1) { vh = h0; ++vt; kb_cur = vt == last_t ? kb_last : kb_full; }
        }
    }
};

// A query block that holds padding only: its rows of a tile-ordered output are zero, a raster
// output has no such rows.  BS: block size, NTHR: threads of the workgroup.
template <int BS, int NTHR>
__device__ __forceinline__ void zero_block_rows(const AttnArgs& a, int bh, int u, int jq) {
    if (a.out_raster) return;
    const int row_bytes = a.out_f32 ? 512 : 256;
    uint4* dst = reinterpret_cast<uint4*>(reinterpret_cast<uint8_t*>(a.out) +
                                          (((size_t)bh * a.g.M + u) * a.g.TSP + (size_t)jq * BS) * row_bytes);
    for (int i = threadIdx.x; i < BS * (row_bytes / 16); i += NTHR) dst[i] = make_uint4(0, 0, 0, 0);
}

// Validity of the BS slots of block jb of sub-tile js of a tile of class cls as wave-wide ballots:
// bit i of word h says whether slot 64h + i of the block is a real token.  Evaluated
// arithmetically, so that tiles of any size need no table.
template <int BS>
__device__ __forceinline__ void block_ballots(const Geom& G, int cls, int js, int jb, int lane,
                                              uint64_t (&bm)[(BS + 63) / 64]) {
    const SubTile so = sub_tile_origin(G, js);
#pragma unroll
    for (int h = 0; h < (BS + 63) / 64; ++h)
        bm[h] = __ballot(sub_slot_is_token(G, cls, so, jb * BS + 64 * h + lane));
}

__device__ __forceinline__ v8i make_v8i(const uint4& lo, const uint4& hi) {
    return v8i{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
}

// Linear HBM -> LDS copy of one 16-byte chunk per lane, done by the load unit itself: lane i of the
// wave deposits its chunk at lds_wave_base + 16 i.  Written as inline assembly so that the
// compiler's wait-count bookkeeping does not serialise it against LDS reads of OTHER buffers; the
// kernel waits for it explicitly (s_waitcnt vmcnt(0)) before the barrier that publishes the tile.
// gsrc is a wave-uniform base (kept in scalar registers), lane_off the lane's byte offset from it.
// OFF (0, 1024, 2048 or 3072) is the instruction's immediate offset: the hardware adds it to the
// global address AND to the LDS address, so the four 1 KB pieces of a wave's 4 KB share of a tile
// need one scalar base each side.
template <int OFF>
__device__ __forceinline__ void dma_chunk(const void* gsrc, uint32_t lane_off, uint32_t lds_wave_base) {
    // both are wave-uniform by construction; say so where the compiler cannot prove it
    const uint64_t p = reinterpret_cast<uint64_t>(gsrc);
    gsrc = reinterpret_cast<const void*>(
        (uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)p) |
        ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(p >> 32)) << 32));
    lds_wave_base = __builtin_amdgcn_readfirstlane(lds_wave_base);
    asm volatile("s_mov_b32 m0, %2\n\t"
                 "s_nop 0\n\t"
                 "global_load_lds_dwordx4 %0, %1 offset:%3"
                 :
                 : "v"(lane_off), "s"(gsrc), "s"(lds_wave_base), "n"(OFF)
                 : "memory", "m0");
}
// chunk c of a wave's contiguous share: base moves every four chunks, the rest rides in the offset
__device__ __forceinline__ void dma_chunk_of(int c, const uint8_t* gsrc_wave, uint32_t lane_off, uint32_t lds_wave) {
    const uint8_t* gs = gsrc_wave + (c >> 2) * 4096;
    const uint32_t ld = lds_wave + (c >> 2) * 4096;
    switch (c & 3) {
        case 0: dma_chunk<0>(gs, lane_off, ld); break;
        case 1: dma_chunk<1024>(gs, lane_off, ld); break;
        case 2: dma_chunk<2048>(gs, lane_off, ld); break;
        default: dma_chunk<3072>(gs, lane_off, ld); break;
    }
}

// The FP8 kernel is software-pipelined inside each wave, because on this chip a wave whose next
// instruction is an MFMA holds the vector issue port while the matrix pipe is busy: MFMA and VALU
// work overlap well only when they alternate within one instruction stream.  Per key tile i:
//   phase 1: row maxima of S(i) (VALU)            interleaved with  O += s^V (V^T P^T)(i-1) (MFMA)
//   phase 2: P(i) = 2^(S'(i) - m), FP8 pack (VALU) interleaved with  S(i+1) = K(i+1) Q^T     (MFMA)
// so the PV product of a tile runs one iteration late and the QK product one iteration early; a
// score block's registers are recycled for the next tile as soon as its exponentials are taken.
// K(i+2) and V(i) stream into LDS during iteration i; one barrier per iteration.
// VCH: V carries one scale per channel (the paper's variant) instead of one per tile; the PV MFMA
// then accumulates straight into O and the scales are applied once in the epilogue.
// NK: what the host knows of the number of key blocks a work item walks -- kOneKeyBlock (every
// item exactly one), kManyKeyBlocks (every item at least two), kAnyKeyBlocks.  With one-block
// tiles it is one or the other for the whole launch; compiling the two cases apart keeps the
// single-block path from joining the pipelined one (the join costs a dozen registers that the
// compiler then spills to scratch memory across the whole main loop: 0.2 GB of HBM writes per call
// at the 720p shape).
enum { kAnyKeyBlocks = 0, kOneKeyBlock = 1, kManyKeyBlocks = 2 };
template <int BS, bool VCH, bool MB, int NK>
__global__ __launch_bounds__(BS * 2) __attribute__((amdgpu_waves_per_eu(2, 2)))
void attn_fp8_kernel(AttnArgs a, MaskTables) {
    constexpr int NB = BS / 16;
    constexpr int NTHR = BS * 2;
    constexpr int CPT = (BS * 8) / NTHR;                   // 16-byte chunks per thread per operand tile
    constexpr bool K_IN_PHASE2 = CPT <= NB;                // K's staging copies ride in phase 2 when its steps suffice
    constexpr int TILE_BYTES = BS * 128;
    __shared__ __attribute__((aligned(16))) uint8_t lds[4][TILE_BYTES];   // K even, K odd, V even, V odd
    const Geom& G = a.g;
    const int KB = MB ? G.KB : 1;                          // blocks per tile; 1 is a compile-time fact
    const int KB_LAST = MB ? G.kb_last : 1;                // ... of a last-along-T tile, without padding-only blocks
    const int KBS = MB ? G.KBS : 1;                        // blocks per quantisation sub-tile (scale group)
    const int NS = MB ? G.NS : 1;                          // sub-tiles per tile
    int bh, u, jq;
    if (!work_item(a, KB, &bh, &u, &jq)) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 4, n = lane & 15;
    const int uw = u % G.nW, uh = (u / G.nW) % G.nH, ut = u / (G.nW * G.nH);
    if (MB && jq >= (ut == G.nT - 1 ? KB_LAST : KB)) {      // a query block of padding only
        zero_block_rows<BS, BS * 2>(a, bh, u, jq);
        return;
    }
    const size_t tile0 = (size_t)bh * G.M;
    const uint32_t lds_base = (uint32_t)(uintptr_t)(&lds[0][0]);   // LDS byte address of buffer 0

    v8i qop[2];
    float m_run[2] = {-INFINITY, -INFINITY};
    float l_run[2] = {0.f, 0.f};                           // running sum of 448 * P
    float alpha_prev[2] = {1.f, 1.f};                      // VCH: rescale owed to O before the delayed PV
    // Per-tile V scales: O and l are kept relative to a FIXED reference m_base (that of the first
    // tile) and each tile's contribution is weighted by 2^(m - m_base) >= 1 instead -- the weight
    // rides in the multiplier of the fma that applies s^V anyway, so a moving row reference costs
    // nothing (rescaling O costs 64 multiplications per wave whenever ANY of its 32 rows moves,
    // which is two tiles in three).  Powers of two commute with fp32 rounding: same results.
    float m_base[2] = {0.f, 0.f};
    float w_cur[2] = {1.f, 1.f};                           // 2^(m - m_base) of the tile whose softmax is taken
    float w_prev[2] = {0.f, 0.f};                          // s^V * 2^(m - m_base) of the tile whose PV is owed
    v4f acc[2][8];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const int row = wave * 32 + qb * 16 + n;
        const uint4* p = reinterpret_cast<const uint4*>(
            a.q + (((tile0 + u) * KB + jq) * BS + row) * 128 + 32 * g);
        qop[qb] = make_v8i(p[0], p[1]);
#pragma unroll
        for (int cb = 0; cb < 8; ++cb) acc[qb][cb] = v4f{0.f, 0.f, 0.f, 0.f};
    }
    const float sqc = load_uniform(a.sq, (tile0 + u) * NS + jq / KBS) * kLog2eOverSqrtD;

    TileWalk w0, w2;                                       // tile i, and the tile whose K is fetched (i+2)
    w0.init(a, KB, KB_LAST, KBS, ut, uh, uw);
    w2 = w0;
    const int ntiles = w0.n;
    auto tile_of = [&](const TileWalk& w) FPS_INLINE { return (w.vt * G.nH + w.vh) * G.nW + w.vw; };

    // chunk c (of CPT) of this thread's share of one operand tile, HBM -> lds[buf]
    const int wave_s = __builtin_amdgcn_readfirstlane(wave);   // the wave index, in a scalar register
    auto stage_chunk = [&](int buf, const uint8_t* src, int c) FPS_INLINE {   // wave w copies bytes [w, w+1) * CPT KB
        dma_chunk_of(c, src + wave_s * (CPT * 1024), lane * 16, lds_base + buf * TILE_BYTES + wave_s * (CPT * 1024));
    };
    auto stage = [&](int buf, const uint8_t* src) FPS_INLINE {
#pragma unroll
        for (int c = 0; c < CPT; ++c) stage_chunk(buf, src, c);
    };
    auto k_blk = [&](const TileWalk& w) FPS_INLINE { return a.k + ((tile0 + tile_of(w)) * KB + w.jk) * TILE_BYTES; };
    auto v_blk = [&](const TileWalk& w) FPS_INLINE { return a.v + ((tile0 + tile_of(w)) * KB + w.jk) * TILE_BYTES; };

    v4f s[2][NB];
    v8i pb[2];                                             // P^T as packed E4M3, 4 keys per dword
    pb[0] = v8i{0, 0, 0, 0, 0, 0, 0, 0};
    pb[1] = pb[0];

    auto load_k = [&](const uint8_t* ldsK, int b) FPS_INLINE {
        const uint4* k4 = reinterpret_cast<const uint4*>(ldsK);
        return make_v8i(k4[(b * 2 + 0) * 64 + lane], k4[(b * 2 + 1) * 64 + lane]);
    };
    auto qk_mfma = [&](const v8i& kop, int b) FPS_INLINE {            // S(b) = K(b) Q^T for both query blocks
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
            s[qb][b] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(
                kop, qop[qb], v4f{0.f, 0.f, 0.f, 0.f}, 0, 0, 0, 0, 0, 0);
    };
    auto load_v = [&](const uint8_t* ldsV, int cb) FPS_INLINE {
        if constexpr (BS == 128) {
            const uint4* v4 = reinterpret_cast<const uint4*>(ldsV);
            return make_v8i(v4[(cb * 2 + 0) * 64 + lane], v4[(cb * 2 + 1) * 64 + lane]);
        } else {
            const uint2 x = reinterpret_cast<const uint2*>(ldsV)[cb * 64 + lane];
            return v8i{(int)x.x, (int)x.y, 0, 0, 0, 0, 0, 0};
        }
    };
    // V^T(cb) P^T for both query blocks: raw into t (per-tile V scales) or accumulated into O (VCH)
    auto pv_mfma = [&](const v8i& vop, v4f (&t)[2], int cb) FPS_INLINE {
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            const v4f c_in = VCH ? acc[qb][cb] : v4f{0.f, 0.f, 0.f, 0.f};
            v4f r;
            if constexpr (BS == 128) {
                r = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(vop, pb[qb], c_in, 0, 0, 0, 0, 0, 0);
            } else {
                const long va = (long)(uint32_t)vop[0] | ((long)(uint32_t)vop[1] << 32);
                const long pa = (long)(uint32_t)pb[qb][0] | ((long)(uint32_t)pb[qb][1] << 32);
                r = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(va, pa, c_in, 0, 0, 0);
            }
            if (VCH) acc[qb][cb] = r; else t[qb] = r;
        }
    };
    // O^T(cb) += s^V * t, pinned where it is written so that t does not stay live (the compiler
    // otherwise sinks all sixteen updates below the loop and spills)
    auto pv_accumulate = [&](int cb, const v4f (&t)[2], const float (&w)[2]) FPS_INLINE {
        if (VCH) return;
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            acc[qb][cb] += t[qb] * w[qb];
            asm volatile("" : "+v"(acc[qb][cb]));
        }
    };
    auto mask_scores = [&](int cls, int js, int jb) FPS_INLINE {      // padded keys of a boundary tile: -inf
        cls = __builtin_amdgcn_readfirstlane(cls);         // wave-uniform by construction
        if (!((a.partial_cls >> cls) & 1u)) return;
        if (!MB) {
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const uint64_t lm = arg_lane_mask(cls, 4 * b + r);   // uniform: one scalar load
                    s[0][b][r] = select_lanes(lm, s[0][b][r], -INFINITY);
                    s[1][b][r] = select_lanes(lm, s[1][b][r], -INFINITY);
                }
        } else {                                           // block jk of a larger tile
            uint64_t bm[(BS + 63) / 64];
            block_ballots<BS>(G, cls, js, jb, lane, bm);
            bool all = true;
#pragma unroll
            for (int h = 0; h < (BS + 63) / 64; ++h) all = all && (bm[h] | (BS >= 64 ? 0ull : ~0xFFFFFFFFull)) == ~0ull;
            if (all) return;                               // most blocks of a boundary tile are whole
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const uint32_t bits = ((uint32_t)(bm[(16 * b) >> 6] >> ((16 * b) & 63)) & 0xFFFFu) >> (4 * g);
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (!((bits >> r) & 1u)) { s[0][b][r] = -INFINITY; s[1][b][r] = -INFINITY; }
            }
        }
    };
    auto rescale_acc = [&]() FPS_INLINE {                             // VCH only
        if (!VCH) return;
        if (__any(alpha_prev[0] != 1.0f || alpha_prev[1] != 1.0f)) {
#pragma unroll
            for (int qb = 0; qb < 2; ++qb)
#pragma unroll
                for (int cb = 0; cb < 8; ++cb) acc[qb][cb] *= alpha_prev[qb];
        }
    };

    // prologue: K(0), K(1) staged; S(0) computed
    stage(0, k_blk(w2));
    w2.next();
    if (ntiles > 1) { stage(1, k_blk(w2)); w2.next(); }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
#pragma unroll
    for (int b = 0; b < NB; ++b) qk_mfma(load_k(lds[0], b), b);
    mask_scores(tile_class(G, w0.vt, w0.vh, w0.vw), w0.js, w0.jb);

    float sc_next = sqc * load_uniform(a.sk, (tile0 + tile_of(w0)) * NS + w0.js);   // scales of the coming block
    float sv_next = VCH ? 1.f : load_uniform(a.sv, (tile0 + tile_of(w0)) * NS + w0.js);
    // One iteration.  FIRST: there is no previous tile whose PV is owed.  LAST: there is no next
    // tile whose scores can be started.  Both are compile-time so that the MFMA / VALU interleave
    // of the steady state carries no branches.
    auto iteration = [&](auto first_tag, auto last_tag, int it) FPS_INLINE {
        constexpr bool FIRST = decltype(first_tag)::value;
        constexpr bool LAST = decltype(last_tag)::value;
        const int par = it & 1;
        const uint8_t* knxt = lds[par ^ 1];                // K(i+1)
        const uint8_t* vprev = lds[2 + (par ^ 1)];         // V(i-1)
        const int v = tile_of(w0);
        const float sc = sc_next;
        const float svv = sv_next;
        if (a.visited && bh == 0 && tid == 0 && jq == 0 && w0.jk == 0) a.visited[(size_t)u * G.M + v] = 1;
        __syncthreads();                 // every wave is past QK(i) and PV(i-2); staged tiles are visible
        // the first V operand is requested at once: its LDS latency passes under the scalar work
        // (tile walk, addresses, scale loads) that follows
        v8i vop[2];
        if (!FIRST) vop[0] = load_v(vprev, 0);
        // K(i+2) replaces K(i), V(i) goes to its own buffer; the copies are issued one per step,
        // V's between the MFMAs of phase 1 and K's in phase 2, rather than in one burst (the load
        // unit takes them slowly)
        const bool fetch_k = it + 2 < ntiles;
        const uint8_t* ksrc = fetch_k ? k_blk(w2) : nullptr;
        const uint8_t* vsrc = v_blk(w0);
        if (fetch_k) w2.next();
        w0.next();
        if (!LAST) {                     // scales of tile i+1, needed next iteration
            const size_t gn = (tile0 + tile_of(w0)) * NS + w0.js;
            sc_next = sqc * load_uniform(a.sk, gn);
            if (!VCH) sv_next = load_uniform(a.sv, gn);
        }

        // ---- phase 1: row maxima of S(i)  |  delayed PV(i-1) --------------------------------
        if (!FIRST) rescale_acc();
        float mx[2];
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
            mx[qb] = __builtin_fmaxf(__builtin_fmaxf(s[qb][0][0], s[qb][0][1]),
                                     __builtin_fmaxf(s[qb][0][2], s[qb][0][3]));
        v4f tq[2][2];                                      // MFMA results wait one block for their fma
#pragma unroll
        for (int cb = 0; cb < 8; ++cb) {
            if (!FIRST) {
                if (cb + 1 < 8) vop[(cb + 1) & 1] = load_v(vprev, cb + 1);
                pv_mfma(vop[cb & 1], tq[cb & 1], cb);
                if (cb > 0) pv_accumulate(cb - 1, tq[(cb - 1) & 1], w_prev);
            }
            if (cb >= 1 && cb < NB) {
#pragma unroll
                for (int qb = 0; qb < 2; ++qb) {
                    mx[qb] = __builtin_fmaxf(__builtin_fmaxf(mx[qb], s[qb][cb][0]), s[qb][cb][1]);
                    mx[qb] = __builtin_fmaxf(__builtin_fmaxf(mx[qb], s[qb][cb][2]), s[qb][cb][3]);
                }
            }
            if (cb < CPT) stage_chunk(2 + par, vsrc, cb);
            else if (!K_IN_PHASE2 && cb < 2 * CPT && fetch_k) stage_chunk(par, ksrc, cb - CPT);
            __builtin_amdgcn_sched_barrier(0);
        }
        static_assert(2 * CPT <= 8, "at most one staging copy per step of a phase");
        if (!FIRST) pv_accumulate(7, tq[1], w_prev);
        v8i kop[2];                      // K(i+1) has been visible since the barrier: ask for its first
        if (!LAST) kop[0] = load_k(knxt, 0);   // operand before the cross-lane reduction of the maxima
        float cm[2];
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            float t = mx[qb];
            t = max_over_row_lanes(t);
            const float m_new = __builtin_fmaxf(m_run[qb], __builtin_ceilf(t * sc));
            if (VCH) {
                alpha_prev[qb] = fast_exp2(m_run[qb] - m_new);
            } else {
                if (FIRST) m_base[qb] = m_new;
                w_cur[qb] = fast_exp2(m_new - m_base[qb]);
            }
            m_run[qb] = m_new;
            // 448 * 2^(S' - m) = 2^(S' + (log2(448) - m)): the factor 448 rides in the exponent
            cm[qb] = kLog2Of448 - m_new;
        }
        // O (complete up to tile i-1 here) and l move to a new reference only when a row has drifted
        // kMaxDrift above its own: 448 * sum|v| * 2^kMaxDrift stays far inside the fp32 range
        if (!VCH && !FIRST &&
            __any(m_run[0] - m_base[0] > kMaxDrift || m_run[1] - m_base[1] > kMaxDrift)) {
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                const float down = fast_exp2(m_base[qb] - m_run[qb]);
#pragma unroll
                for (int cb = 0; cb < 8; ++cb) acc[qb][cb] *= down;
                l_run[qb] *= down;
                m_base[qb] = m_run[qb];
                w_cur[qb] = 1.0f;
            }
        }

        // ---- phase 2: P(i) and its FP8 codes  |  early QK(i+1) ------------------------------
        float rs[2] = {0.f, 0.f};
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            if (!LAST && b + 1 < NB) kop[(b + 1) & 1] = load_k(knxt, b + 1);
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                float p[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    p[r] = fast_exp2(__builtin_fmaf(s[qb][b][r], sc, cm[qb]));
                    rs[qb] += p[r];
                }
                int pw = pb[qb][b];                        // both halves are overwritten below
                pw = __builtin_amdgcn_cvt_pk_fp8_f32(p[0], p[1], pw, false);
                pw = __builtin_amdgcn_cvt_pk_fp8_f32(p[2], p[3], pw, true);
                // pinned here: otherwise the compiler sinks the whole exponential pass below the
                // MFMAs it is meant to overlap with
                asm volatile("" : "+v"(pw), "+v"(rs[qb]));
                pb[qb][b] = pw;
            }
            if (!LAST) qk_mfma(kop[b & 1], b);
            if (K_IN_PHASE2 && b < CPT && fetch_k) stage_chunk(par, ksrc, b);   // K(i) was consumed last iteration
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            if (VCH) l_run[qb] = l_run[qb] * alpha_prev[qb] + rs[qb];
            else     l_run[qb] = __builtin_fmaf(rs[qb], w_cur[qb], l_run[qb]);
            w_prev[qb] = svv * w_cur[qb];
        }
        if (!LAST) mask_scores(tile_class(G, w0.vt, w0.vh, w0.vw), w0.js, w0.jb);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this thread's share of the staged tiles landed
    };
    using T_ = std::true_type;
    using F_ = std::false_type;
    if constexpr (NK == kOneKeyBlock) {
        iteration(T_{}, T_{}, 0);
    } else if constexpr (NK == kManyKeyBlocks) {
        iteration(T_{}, F_{}, 0);
        for (int it = 1; it + 1 < ntiles; ++it) iteration(F_{}, F_{}, it);
        iteration(F_{}, T_{}, ntiles - 1);
    } else if (ntiles == 1) {
        iteration(T_{}, T_{}, 0);
    } else {
        iteration(T_{}, F_{}, 0);
        for (int it = 1; it + 1 < ntiles; ++it) iteration(F_{}, F_{}, it);
        iteration(F_{}, T_{}, ntiles - 1);
    }
    // epilogue: the last tile's PV
    __syncthreads();
    rescale_acc();
    {
        const uint8_t* vlast = lds[2 + ((ntiles - 1) & 1)];
        v4f tq[2];
#pragma unroll
        for (int cb = 0; cb < 8; ++cb) {
            pv_mfma(load_v(vlast, cb), tq, cb);
            pv_accumulate(cb, tq, w_prev);
        }
    }

    float inv[2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        float l = l_run[qb];
        l = sum_over_row_lanes(l);
        inv[qb] = l > 0.f ? 1.0f / l : 0.f;               // l already carries the factor 448
    }
    __syncthreads();                                       // all waves are done with the staged tiles
    store_rows<BS>(a, bh, u, jq, KBS, tile_class(G, ut, uh, uw), wave, lane, acc, inv,
                   &lds[0][0] + wave * kStoreRegionBytes, VCH ? a.sv + (size_t)bh * 128 : nullptr);
}

// ---------------------------------------------------------------------------------------------
// FP8, 128-slot blocks: the same pipeline on v_mfma_f32_32x32x64_f8f6f4.  One instruction of 16
// passes does the work of two 16x16x128 ones, and what an MFMA costs the vector instructions
// around it is largely per instruction (measured with fps_debug_issue_mix: beside 32 vector
// instructions one 32x32x64 adds 30 clocks, two 16x16x128 add 49), so the softmax's vector work
// shares the SIMD with half as many matrix instructions.  A wave owns 32 query rows as ONE operand
// block: lane (n, h) = lane & 31, lane >> 5 holds query n; of a 32-key score block kb it holds the
// keys 8(r/4) + 4h + r%4, r = 0..15; of a 32-channel output block db the channels of the same
// pattern.  The other lane of the row is lane n + 32.
// ---------------------------------------------------------------------------------------------
typedef float v16f __attribute__((ext_vector_type(16)));

__device__ __forceinline__ v16f zero16() {
    v16f z;
#pragma unroll
    for (int r = 0; r < 16; ++r) z[r] = 0.f;
    return z;
}
__device__ __forceinline__ float max_over_row_pair(float t) {          // lanes n and n + 32
    const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(t), __float_as_uint(t), false, false);
    return __builtin_fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_over_row_pair(float t) {
    const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(t), __float_as_uint(t), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
// x if bit `idx` of the lane's word `bits` is set, otherwise -inf: two vector instructions (a
// sign-extended one-bit field, a bitwise select) and no compare, so a run of them needs no scalar
// registers for compare results
__device__ __forceinline__ float keep_if_bit(float x, uint32_t bits, int idx) {
    const uint32_t m = (uint32_t)(-(int)((bits >> idx) & 1u));
    return __uint_as_float((__float_as_uint(x) & m) | (0xFF800000u & ~m));
}
// pair_code[c][kb], bits 2r + h: set iff the key that lane half h holds in register r of score block
// kb, slot 32kb + 8(r/4) + 4h + r%4 of a one-block tile of class c, is a real token
__device__ __forceinline__ uint32_t arg_pair_code(int cls, int kb) {
    typedef const __attribute__((address_space(4))) uint32_t* ptr_t;
    const __attribute__((address_space(4))) char* base =
        (const __attribute__((address_space(4))) char*)__builtin_amdgcn_kernarg_segment_ptr();
    return ((ptr_t)(base + kTablesOffset + offsetof(MaskTables, pair_code)))[cls * 4 + kb];
}
// the wave-wide lane mask of register r: all of a lane half, or none of it
__device__ __forceinline__ uint64_t pair_lane_mask(uint32_t code, int r) {
    const uint32_t c2 = code >> (2 * r);
    return (uint64_t)(uint32_t)(-(int)(c2 & 1u)) | ((uint64_t)(uint32_t)(-(int)((c2 >> 1) & 1u)) << 32);
}

// Epilogue of the wide kernel: as store_rows, for accumulators of the 32x32 shape.  The wave's 32
// rows go through its LDS region in two passes of 16 rows (rows n < 16 are held by lanes 0..15 and
// 32..47).
__device__ __forceinline__ void store_rows_wide(const AttnArgs& a, int bh, int u, int jq, int KBS, int ucls,
                                                int wave, int lane, const v16f (&acc)[4], float inv,
                                                uint8_t* wave_lds, const float* ch_scale = nullptr) {
    constexpr int BS = 128;
    const auto& G = a.g;
    const int h = lane >> 5, n = lane & 31;
    const int row_bytes = a.out_f32 ? 512 : 256;
    const int pitch = row_bytes + 16;
    const int uw = u % G.nW, uh = (u / G.nW) % G.nH, ut = u / (G.nW * G.nH);
    const int sub = jq / KBS;
    const SubTile so = sub_tile_origin(G, sub);
    const int slot0 = (jq - sub * KBS) * BS;
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        if ((n >> 4) == pass) {
            const int rr = n & 15;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    const int col = 32 * db + 8 * q4 + 4 * h;
                    v4f o = v4f{acc[db][4 * q4], acc[db][4 * q4 + 1], acc[db][4 * q4 + 2], acc[db][4 * q4 + 3]} * inv;
                    if (ch_scale) o *= *reinterpret_cast<const v4f*>(ch_scale + col);
                    if (a.out_f32) {
                        *reinterpret_cast<v4f*>(wave_lds + rr * pitch + col * 4) = o;
                    } else {
                        uint2 pk;
                        pk.x = pack_bf16x2(o[0], o[1]);
                        pk.y = pack_bf16x2(o[2], o[3]);
                        *reinterpret_cast<uint2*>(wave_lds + rr * pitch + col * 2) = pk;
                    }
                }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        const int lanes_shift = a.out_f32 ? 5 : 4;
        const int rows_per_pass = 64 >> lanes_shift;
        for (int r0 = 0; r0 < 16; r0 += rows_per_pass) {
            const int r = r0 + (lane >> lanes_shift), chunk = lane & ((1 << lanes_shift) - 1);
            const int in_block = wave * 32 + pass * 16 + r;
            int rt = 0, rh = 0, rw = 0;
            const bool valid = sub_slot_coords(G, so, slot0 + in_block, &rt, &rh, &rw) &&
                               coords_in_class(G, ucls, rt, rh, rw);
            uint4 val = *reinterpret_cast<const uint4*>(wave_lds + r * pitch + chunk * 16);
            size_t row;
            if (a.out_raster) {
                if (!valid) continue;
                row = (((size_t)bh * G.T + (ut * G.Tt + rt)) * G.H + (uh * G.Th + rh)) * G.W + (uw * G.Tw + rw);
            } else {
                row = ((size_t)bh * G.M + u) * G.TSP + (size_t)jq * BS + in_block;
                if (!valid) val = make_uint4(0, 0, 0, 0);
            }
            reinterpret_cast<uint4*>(reinterpret_cast<uint8_t*>(a.out) + row * row_bytes)[chunk] = val;
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
}

template <bool VCH, bool MB, int NK>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
void attn_fp8_wide_kernel(AttnArgs a, MaskTables) {
    constexpr int BS = 128;
    constexpr int NTHR = 256;
    constexpr int CPT = (BS * 8) / NTHR;                   // 16-byte chunks per thread per operand tile (4)
    constexpr int TILE_BYTES = BS * 128;
    __shared__ __attribute__((aligned(16))) uint8_t lds[4][TILE_BYTES];   // K even, K odd, V even, V odd
    const Geom& G = a.g;
    const int KB = MB ? G.KB : 1;
    const int KB_LAST = MB ? G.kb_last : 1;
    const int KBS = MB ? G.KBS : 1;
    const int NS = MB ? G.NS : 1;
    int bh, u, jq;
    if (!work_item(a, KB, &bh, &u, &jq)) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, h = lane >> 5, n = lane & 31;
    const int uw = u % G.nW, uh = (u / G.nW) % G.nH, ut = u / (G.nW * G.nH);
    if (MB && jq >= (ut == G.nT - 1 ? KB_LAST : KB)) {      // a query block of padding only
        zero_block_rows<BS, NTHR>(a, bh, u, jq);
        return;
    }
    const size_t tile0 = (size_t)bh * G.M;
    const uint32_t lds_base = (uint32_t)(uintptr_t)(&lds[0][0]);

    v8i qop[2];                                            // Q^T, contraction steps 0 and 1
    float m_run = -INFINITY;
    float l_run = 0.f;                                     // running sum of 448 * P (this lane's keys)
    float alpha_prev = 1.f;                                // VCH: rescale owed to O before the delayed PV
    float m_base = 0.f, w_cur = 1.f, w_prev = 0.f;         // fixed reference and weights: see attn_fp8_kernel
    v16f acc[4];
    {
        const int row = wave * 32 + n;
        const uint4* p = reinterpret_cast<const uint4*>(
            a.q + (((tile0 + u) * KB + jq) * BS + row) * 128 + 32 * h);
        qop[0] = make_v8i(p[0], p[1]);
        qop[1] = make_v8i(p[4], p[5]);
#pragma unroll
        for (int db = 0; db < 4; ++db) acc[db] = zero16();
    }
    const float sqc = load_uniform(a.sq, (tile0 + u) * NS + jq / KBS) * kLog2eOverSqrtD;

    TileWalk w0, w2;
    w0.init(a, KB, KB_LAST, KBS, ut, uh, uw);
    w2 = w0;
    const int ntiles = w0.n;
    auto tile_of = [&](const TileWalk& w) FPS_INLINE { return (w.vt * G.nH + w.vh) * G.nW + w.vw; };
    const int wave_s = __builtin_amdgcn_readfirstlane(wave);
    auto stage_chunk = [&](int buf, const uint8_t* src, int c) FPS_INLINE {
        dma_chunk_of(c, src + wave_s * (CPT * 1024), lane * 16, lds_base + buf * TILE_BYTES + wave_s * (CPT * 1024));
    };
    auto stage = [&](int buf, const uint8_t* src) FPS_INLINE {
#pragma unroll
        for (int c = 0; c < CPT; ++c) stage_chunk(buf, src, c);
    };
    auto k_blk = [&](const TileWalk& w) FPS_INLINE { return a.k + ((tile0 + tile_of(w)) * KB + w.jk) * TILE_BYTES; };
    auto v_blk = [&](const TileWalk& w) FPS_INLINE { return a.v + ((tile0 + tile_of(w)) * KB + w.jk) * TILE_BYTES; };

    v16f s[4];                                             // S^T, four blocks of 32 keys
    v8i pb[2];                                             // P^T as packed E4M3: contraction steps 0 and 1
    pb[0] = v8i{0, 0, 0, 0, 0, 0, 0, 0};
    pb[1] = pb[0];

    // operand `step` (block * 2 + contraction step) of a staged K or V block
    auto load_op = [&](const uint8_t* buf, int step) FPS_INLINE {
        const uint4* b4 = reinterpret_cast<const uint4*>(buf);
        return make_v8i(b4[(step * 2 + 0) * 64 + lane], b4[(step * 2 + 1) * 64 + lane]);
    };
    auto qk_mfma = [&](const v8i& kop, int step) FPS_INLINE {
        const int kb = step >> 1, ks = step & 1;
        s[kb] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(kop, qop[ks], ks == 0 ? zero16() : s[kb],
                                                               0, 0, 0, 0, 0, 0);
    };
    v16f tq[2];                                            // raw V^T P^T of a channel block, until its fma
    auto pv_mfma = [&](const v8i& vop, int step) FPS_INLINE {
        const int db = step >> 1, j = step & 1;
        if (VCH) acc[db] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(vop, pb[j], acc[db], 0, 0, 0, 0, 0, 0);
        else     tq[db & 1] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                     vop, pb[j], j == 0 ? zero16() : tq[db & 1], 0, 0, 0, 0, 0, 0);
    };
    // half `half` of O^T(db) += s^V 2^(m - m_base) * raw, pinned where it is written
    auto pv_accumulate_half = [&](int db, int half) FPS_INLINE {
        if (VCH) return;
#pragma unroll
        for (int r = 8 * half; r < 8 * half + 8; ++r) acc[db][r] = __builtin_fmaf(tq[db & 1][r], w_prev, acc[db][r]);
        asm volatile("" : "+v"(acc[db]));
    };
    auto mask_scores = [&](int cls, int js, int jb) FPS_INLINE {      // padded keys of a boundary tile: -inf
        cls = __builtin_amdgcn_readfirstlane(cls);
        if (!((a.partial_cls >> cls) & 1u)) return;
        if (!MB) {
#pragma unroll
            for (int kb = 0; kb < 4; ++kb) {
                const uint32_t code = arg_pair_code(cls, kb);          // uniform: one scalar load
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    s[kb][r] = select_lanes(pair_lane_mask(code, r), s[kb][r], -INFINITY);
            }
        } else {
            uint64_t bm[2];
            block_ballots<BS>(G, cls, js, jb, lane, bm);
            if ((bm[0] & bm[1]) == ~0ull) return;          // most blocks of a boundary tile are whole
#pragma unroll
            for (int kb = 0; kb < 4; ++kb) {
                const uint32_t bits = (uint32_t)(bm[kb >> 1] >> (32 * (kb & 1))) >> (4 * h);
#pragma unroll
                for (int r = 0; r < 16; ++r) s[kb][r] = keep_if_bit(s[kb][r], bits, 8 * (r >> 2) + (r & 3));
            }
        }
    };
    auto rescale_acc = [&]() FPS_INLINE {                             // VCH only
        if (!VCH) return;
        if (__any(alpha_prev != 1.0f)) {
#pragma unroll
            for (int db = 0; db < 4; ++db) acc[db] *= alpha_prev;
        }
    };

    // prologue: K(0), K(1) staged; S(0) computed
    stage(0, k_blk(w2));
    w2.next();
    if (ntiles > 1) { stage(1, k_blk(w2)); w2.next(); }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
#pragma unroll
    for (int step = 0; step < 8; ++step) qk_mfma(load_op(lds[0], step), step);
    mask_scores(tile_class(G, w0.vt, w0.vh, w0.vw), w0.js, w0.jb);

    float sc_next = sqc * load_uniform(a.sk, (tile0 + tile_of(w0)) * NS + w0.js);
    float sv_next = VCH ? 1.f : load_uniform(a.sv, (tile0 + tile_of(w0)) * NS + w0.js);
    auto iteration = [&](auto first_tag, auto last_tag, int it) FPS_INLINE {
        constexpr bool FIRST = decltype(first_tag)::value;
        constexpr bool LAST = decltype(last_tag)::value;
        const int par = it & 1;
        const uint8_t* knxt = lds[par ^ 1];                // K(i+1)
        const uint8_t* vprev = lds[2 + (par ^ 1)];         // V(i-1)
        const int v = tile_of(w0);
        const float sc = sc_next;
        const float svv = sv_next;
        if (a.visited && bh == 0 && tid == 0 && jq == 0 && w0.jk == 0) a.visited[(size_t)u * G.M + v] = 1;
        __syncthreads();                 // every wave is past QK(i) and PV(i-2); staged tiles are visible
        v8i op[3];                       // MFMA operands on their way from LDS, two steps ahead
        if (!FIRST) { op[0] = load_op(vprev, 0); op[1] = load_op(vprev, 1); }
        const bool fetch_k = it + 2 < ntiles;
        const uint8_t* ksrc = fetch_k ? k_blk(w2) : nullptr;
        const uint8_t* vsrc = v_blk(w0);
        if (fetch_k) w2.next();
        w0.next();
        if (!LAST) {                     // scales of tile i+1, needed next iteration
            const size_t gn = (tile0 + tile_of(w0)) * NS + w0.js;
            sc_next = sqc * load_uniform(a.sk, gn);
            if (!VCH) sv_next = load_uniform(a.sv, gn);
        }

        // ---- phase 1: row maximum of S(i)  |  delayed PV(i-1) --------------------------------
        // step k: half the fma of the block whose second MFMA was issued two or three steps earlier
        // (a 16-pass result may be read 18 issue slots after its instruction), the MFMA of channel
        // block k/2, contraction step k%2, and an eighth of the row maximum
        if (!FIRST) rescale_acc();
        float mx = __builtin_fmaxf(__builtin_fmaxf(s[0][0], s[0][1]), __builtin_fmaxf(s[0][2], s[0][3]));
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            if (!FIRST) {
                if (k + 2 < 8) op[(k + 2) % 3] = load_op(vprev, k + 2);
                if (k >= 3) pv_accumulate_half((k - 3) >> 1, (k - 3) & 1);   // before tq[..] is refilled
                pv_mfma(op[k % 3], k);
            }
#pragma unroll
            for (int r = (k == 0 ? 4 : 8 * (k & 1)); r < 8 * (k & 1) + 8; r += 2)
                mx = __builtin_fmaxf(__builtin_fmaxf(mx, s[k >> 1][r]), s[k >> 1][r + 1]);
            asm volatile("" : "+v"(mx));
            if (k < CPT) stage_chunk(2 + par, vsrc, k);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (!FIRST) pv_accumulate_half(2, 1);
        if (!LAST) { op[0] = load_op(knxt, 0); op[1] = load_op(knxt, 1); }   // K(i+1): visible since the barrier
        mx = max_over_row_pair(mx);
        const float m_new = __builtin_fmaxf(m_run, __builtin_ceilf(mx * sc));
        if (VCH) {
            alpha_prev = fast_exp2(m_run - m_new);
        } else {
            if (FIRST) m_base = m_new;
            w_cur = fast_exp2(m_new - m_base);
        }
        m_run = m_new;
        const float cm = kLog2Of448 - m_new;   // 448 * 2^(S' - m) = 2^(S' + (log2(448) - m))
        if (!VCH && !FIRST && __any(m_run - m_base > kMaxDrift)) {
            const float down = fast_exp2(m_base - m_run);
#pragma unroll
            for (int db = 0; db < 4; ++db) acc[db] *= down;
            l_run *= down;
            w_prev *= down;              // the last channel block's fma is still owed (steps 0, 1 below)
            m_base = m_run;
            w_cur = 1.0f;
        }

        // ---- phase 2: P(i) and its FP8 codes  |  early QK(i+1) ------------------------------
        // step t: the exponentials of half a score block (block t/2, registers 8(t%2)..+7); the
        // MFMAs that refill a block follow one block behind, so steps 0, 1 have none (they take the
        // fma still owed to the last channel block of PV(i-1)) and steps 8, 9 nothing else
        float rs = 0.f;
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < 10; ++t) {
            if (!LAST && t >= 2) {
                if (t < 8) op[t % 3] = load_op(knxt, t);               // operand of step t + 2
                qk_mfma(op[(t - 2) % 3], t - 2);
            }
            if (!FIRST && t < 2) pv_accumulate_half(3, t);             // PV(i-1)'s last block
            if (t < 8) {
                const int kb = t >> 1, e = t & 1;
#pragma unroll
                for (int q2 = 0; q2 < 2; ++q2) {
                    float p[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        p[r] = fast_exp2(__builtin_fmaf(s[kb][8 * e + 4 * q2 + r], sc, cm));
                        rs += p[r];
                    }
                    int pw = pb[kb >> 1][4 * (kb & 1) + 2 * e + q2];
                    pw = __builtin_amdgcn_cvt_pk_fp8_f32(p[0], p[1], pw, false);
                    pw = __builtin_amdgcn_cvt_pk_fp8_f32(p[2], p[3], pw, true);
                    asm volatile("" : "+v"(pw), "+v"(rs));  // keep the pass where it is written
                    pb[kb >> 1][4 * (kb & 1) + 2 * e + q2] = pw;
                }
            }
            if (t < CPT && fetch_k) stage_chunk(par, ksrc, t);   // K(i) was consumed last iteration
            __builtin_amdgcn_sched_barrier(0);
        }
        if (VCH) l_run = l_run * alpha_prev + rs;
        else     l_run = __builtin_fmaf(rs, w_cur, l_run);
        w_prev = svv * w_cur;
        if (!LAST) mask_scores(tile_class(G, w0.vt, w0.vh, w0.vw), w0.js, w0.jb);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this thread's share of the staged tiles landed
    };
    using T_ = std::true_type;
    using F_ = std::false_type;
    if constexpr (NK == kOneKeyBlock) {
        iteration(T_{}, T_{}, 0);
    } else if constexpr (NK == kManyKeyBlocks) {
        iteration(T_{}, F_{}, 0);
        for (int it = 1; it + 1 < ntiles; ++it) iteration(F_{}, F_{}, it);
        iteration(F_{}, T_{}, ntiles - 1);
    } else if (ntiles == 1) {
        iteration(T_{}, T_{}, 0);
    } else {
        iteration(T_{}, F_{}, 0);
        for (int it = 1; it + 1 < ntiles; ++it) iteration(F_{}, F_{}, it);
        iteration(F_{}, T_{}, ntiles - 1);
    }
    // epilogue: the last tile's PV
    __syncthreads();
    rescale_acc();
    {
        const uint8_t* vlast = lds[2 + ((ntiles - 1) & 1)];
#pragma unroll
        for (int db = 0; db < 4; ++db) {
            pv_mfma(load_op(vlast, 2 * db), 2 * db);
            pv_mfma(load_op(vlast, 2 * db + 1), 2 * db + 1);
            pv_accumulate_half(db, 0);
            pv_accumulate_half(db, 1);
        }
    }
    const float l = sum_over_row_pair(l_run);
    const float inv = l > 0.f ? 1.0f / l : 0.f;            // l already carries the factor 448
    __syncthreads();                                       // all waves are done with the staged tiles
    store_rows_wide(a, bh, u, jq, KBS, tile_class(G, ut, uh, uw), wave, lane, acc, inv,
                    &lds[0][0] + wave * kStoreRegionBytes, VCH ? a.sv + (size_t)bh * 128 : nullptr);
}

// ---------------------------------------------------------------------------------------------
// BF16: no quantisation.  K Q^T on v_mfma_f32_16x16x32_bf16; P is rounded to fp16 and multiplied
// with the fp16 V tiles (exact per-tile power-of-two scaling, undone by s^V) on
// v_mfma_f32_16x16x32_f16.  Same in-wave pipeline as the FP8 kernel (PV one tile late, QK one tile
// early).  A bf16 tile pair is 64 KB, so K and V are single-buffered: K(i+1) streams in during
// phase 1 (after every wave has finished reading K(i)), V(i) during phase 2 (after every wave has
// finished PV(i-1)); two barriers per iteration.
// ---------------------------------------------------------------------------------------------
union Bf16x8 { uint4 u; v8bf v; v8h h; };

template <int BS, bool MB, int NK>
__global__ __launch_bounds__(BS * 2) __attribute__((amdgpu_waves_per_eu(2, 2)))
void attn_bf16_kernel(AttnArgs a, MaskTables) {
    constexpr int NB = BS / 16;
    constexpr int NKK = BS / 32;
    constexpr int NTHR = BS * 2;
    constexpr int TILE_BYTES = BS * 256;
    constexpr int CPT = (BS * 16) / NTHR;                  // 16-byte chunks per thread per operand tile (8)
    __shared__ __attribute__((aligned(16))) uint8_t lds[2][TILE_BYTES];   // K, V
    const Geom& G = a.g;
    const int KB = MB ? G.KB : 1;                          // blocks per tile; 1 is a compile-time fact
    const int KB_LAST = MB ? G.kb_last : 1;                // ... of a last-along-T tile, without padding-only blocks
    const int KBS = MB ? G.KBS : 1;                        // blocks per quantisation sub-tile (scale group)
    const int NS = MB ? G.NS : 1;                          // sub-tiles per tile
    int bh, u, jq;
    if (!work_item(a, KB, &bh, &u, &jq)) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 4, n = lane & 15;
    const int uw = u % G.nW, uh = (u / G.nW) % G.nH, ut = u / (G.nW * G.nH);
    if (MB && jq >= (ut == G.nT - 1 ? KB_LAST : KB)) {      // a query block of padding only
        zero_block_rows<BS, BS * 2>(a, bh, u, jq);
        return;
    }
    const size_t tile0 = (size_t)bh * G.M;
    const uint32_t lds_base = (uint32_t)(uintptr_t)(&lds[0][0]);

    Bf16x8 qop[2][4];
    float m_run[2] = {-INFINITY, -INFINITY};
    float l_run[2] = {0.f, 0.f};
    // O and l relative to the fixed reference m_base, contributions weighted by 2^(m - m_base): see
    // the FP8 kernel
    float m_base[2] = {0.f, 0.f};
    float w_cur[2] = {1.f, 1.f};
    float w_prev[2] = {0.f, 0.f};
    v4f acc[2][8];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const int row = wave * 32 + qb * 16 + n;
        const uint4* p = reinterpret_cast<const uint4*>(a.q + (((tile0 + u) * KB + jq) * BS + row) * 256);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) qop[qb][ks].u = p[ks * 4 + g];
#pragma unroll
        for (int cb = 0; cb < 8; ++cb) acc[qb][cb] = v4f{0.f, 0.f, 0.f, 0.f};
    }
    const float sc = kLog2eOverSqrtD;

    TileWalk w0, w1;                                       // tile i and tile i+1
    w0.init(a, KB, KB_LAST, KBS, ut, uh, uw);
    w1 = w0;
    w1.next();
    const int ntiles = w0.n;
    auto tile_of = [&](const TileWalk& w) FPS_INLINE { return (w.vt * G.nH + w.vh) * G.nW + w.vw; };
    const int wave_s = __builtin_amdgcn_readfirstlane(wave);   // the wave index, in a scalar register
    auto stage_chunk = [&](int buf, const uint8_t* src, int c) FPS_INLINE {   // wave w copies bytes [w, w+1) * CPT KB
        dma_chunk_of(c, src + wave_s * (CPT * 1024), lane * 16, lds_base + buf * TILE_BYTES + wave_s * (CPT * 1024));
    };
    auto k_blk = [&](const TileWalk& w) FPS_INLINE { return a.k + ((tile0 + tile_of(w)) * KB + w.jk) * TILE_BYTES; };
    auto v_blk = [&](const TileWalk& w) FPS_INLINE { return a.v + ((tile0 + tile_of(w)) * KB + w.jk) * TILE_BYTES; };
    const uint4* ldsK4 = reinterpret_cast<const uint4*>(lds[0]);
    const uint4* ldsV4 = reinterpret_cast<const uint4*>(lds[1]);

    v4f s[2][NB];
    Bf16x8 pop[2][NKK];                                    // P^T in fp16, 8 keys per operand
    Bf16x8 ring[4];                                        // MFMA operands on their way from LDS

    auto qk_block = [&](int b) FPS_INLINE {                           // S(b) = K(b) Q^T, both query blocks
        Bf16x8 kop[4];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) kop[ks].u = ldsK4[(b * 4 + ks) * 64 + lane];
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            v4f r = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
                r = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kop[ks].v, qop[qb][ks].v, r, 0, 0, 0);
            s[qb][b] = r;
        }
    };
    auto pv_block = [&](int cb, v4f (&t)[2]) FPS_INLINE {             // V^T(cb) P^T, raw, both query blocks
        Bf16x8 vop[NKK];
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk) vop[kk].u = ldsV4[(kk * 8 + cb) * 64 + lane];
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            v4f r = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < NKK; ++kk)
                r = __builtin_amdgcn_mfma_f32_16x16x32_f16(vop[kk].h, pop[qb][kk].h, r, 0, 0, 0);
            t[qb] = r;
        }
    };
    auto pv_accumulate = [&](int cb, const v4f (&t)[2], const float (&w)[2]) FPS_INLINE {
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            acc[qb][cb] += t[qb] * w[qb];
            asm volatile("" : "+v"(acc[qb][cb]));
        }
    };
    auto mask_scores = [&](int cls, int js, int jb) FPS_INLINE {      // padded keys of a boundary tile: -inf
        cls = __builtin_amdgcn_readfirstlane(cls);         // wave-uniform by construction
        if (!((a.partial_cls >> cls) & 1u)) return;
        if (!MB) {
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const uint64_t lm = arg_lane_mask(cls, 4 * b + r);   // uniform: one scalar load
                    s[0][b][r] = select_lanes(lm, s[0][b][r], -INFINITY);
                    s[1][b][r] = select_lanes(lm, s[1][b][r], -INFINITY);
                }
        } else {                                           // block jk of a larger tile
            uint64_t bm[(BS + 63) / 64];
            block_ballots<BS>(G, cls, js, jb, lane, bm);
            bool all = true;
#pragma unroll
            for (int h = 0; h < (BS + 63) / 64; ++h) all = all && (bm[h] | (BS >= 64 ? 0ull : ~0xFFFFFFFFull)) == ~0ull;
            if (all) return;                               // most blocks of a boundary tile are whole
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const uint32_t bits = ((uint32_t)(bm[(16 * b) >> 6] >> ((16 * b) & 63)) & 0xFFFFu) >> (4 * g);
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (!((bits >> r) & 1u)) { s[0][b][r] = -INFINITY; s[1][b][r] = -INFINITY; }
            }
        }
    };
    // prologue: K(0) staged, S(0) computed
#pragma unroll
    for (int c = 0; c < CPT; ++c) stage_chunk(0, k_blk(w0), c);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
#pragma unroll
    for (int b = 0; b < NB; ++b) qk_block(b);
    mask_scores(tile_class(G, w0.vt, w0.vh, w0.vw), w0.js, w0.jb);

    auto iteration = [&](auto first_tag, auto last_tag) FPS_INLINE {
        constexpr bool FIRST = decltype(first_tag)::value;
        constexpr bool LAST = decltype(last_tag)::value;
        const int v = tile_of(w0);
        const float svv = load_uniform(a.sv, (tile0 + v) * NS + w0.js);
        if (a.visited && bh == 0 && tid == 0 && jq == 0 && w0.jk == 0) a.visited[(size_t)u * G.M + v] = 1;
        const uint8_t* ksrc = LAST ? nullptr : k_blk(w1);
        const uint8_t* vsrc = v_blk(w0);
        __syncthreads();                 // every wave has finished QK(i): the K buffer is free; V(i-1) visible

        // ---- phase 1: row maxima of S(i)  |  delayed PV(i-1)  |  K(i+1) streams in ------------
        // One step per MFMA pair (the two query blocks against one V operand).  The operands come
        // through a ring of four registers, requested three pairs ahead; the vector work of the
        // step -- a quarter of the previous channel block's accumulation and of this block's row
        // maxima -- sits between the two MFMAs.  K's copies are all issued in the first half, so
        // that they have landed when the phase ends.
        float mx[2];
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
            mx[qb] = __builtin_fmaxf(__builtin_fmaxf(s[qb][0][0], s[qb][0][1]),
                                     __builtin_fmaxf(s[qb][0][2], s[qb][0][3]));
        constexpr int NPV = 8 * NKK;                       // pairs of phase 1
        auto v_operand = [&](int j) FPS_INLINE { return ldsV4[((j % NKK) * 8 + j / NKK) * 64 + lane]; };
        v4f tq[2][2];                                      // a block's raw product waits one block for its fma
        // quarter `part` of the vector work that accompanies channel block cb: a row-maximum step,
        // and in quarters 1 and 2 the accumulation of block cb - 1 for one query block (its last
        // MFMA was issued at least two MFMAs earlier, so the fma does not wait for it)
        auto phase1_valu = [&](int cb, int part) FPS_INLINE {
            const int qb = part >> 1, h = part & 1;
            if (cb >= 1 && cb < NB)
                mx[qb] = __builtin_fmaxf(__builtin_fmaxf(mx[qb], s[qb][cb][2 * h]), s[qb][cb][2 * h + 1]);
            if (!FIRST && cb >= 1 && (part == 1 || part == 2)) {
                acc[part - 1][cb - 1] += tq[(cb - 1) & 1][part - 1] * w_prev[part - 1];
                asm volatile("" : "+v"(acc[part - 1][cb - 1]));
            }
        };
        if (!FIRST) {
#pragma unroll
            for (int j = 0; j < 3 && j < NPV; ++j) ring[j].u = v_operand(j);
        }
#pragma unroll
        for (int j = 0; j < NPV; ++j) {
            const int cb = j / NKK, kk = j % NKK;
            if (!FIRST) {
                if (j + 3 < NPV) ring[(j + 3) & 3].u = v_operand(j + 3);
                tq[cb & 1][0] = __builtin_amdgcn_mfma_f32_16x16x32_f16(
                    ring[j & 3].h, pop[0][kk].h, kk == 0 ? v4f{0.f, 0.f, 0.f, 0.f} : tq[cb & 1][0], 0, 0, 0);
            }
#pragma unroll
            for (int part = kk * (4 / NKK); part < (kk + 1) * (4 / NKK); ++part) phase1_valu(cb, part);
            if (!FIRST)
                tq[cb & 1][1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(
                    ring[j & 3].h, pop[1][kk].h, kk == 0 ? v4f{0.f, 0.f, 0.f, 0.f} : tq[cb & 1][1], 0, 0, 0);
            if (kk == NKK - 1) asm volatile("" : "+v"(mx[0]), "+v"(mx[1]));
            if (!LAST && kk == 0 && cb < 4) {
                stage_chunk(0, ksrc, 2 * cb);
                stage_chunk(0, ksrc, 2 * cb + 1);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        if (!FIRST) pv_accumulate(7, tq[1], w_prev);
        static_assert(CPT == 8, "K staging: two chunks in each of the first four channel blocks");
        float cm[2];
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            float t = mx[qb];
            t = max_over_row_lanes(t);
            const float m_new = __builtin_fmaxf(m_run[qb], __builtin_ceilf(t * sc));
            if (FIRST) m_base[qb] = m_new;
            w_cur[qb] = fast_exp2(m_new - m_base[qb]);
            m_run[qb] = m_new;
            // 2^14 * 2^(S' - m): the factor rides in the exponent and cancels against the row sum,
            // which is taken of the same scaled values; it keeps weights down to 2^-28 in fp16's
            // normal range (a dense row over thousands of keys has many weights below 2^-14)
            cm[qb] = kFp16PScaleLog2 - m_new;
        }
        if (!FIRST && __any(m_run[0] - m_base[0] > kMaxDrift || m_run[1] - m_base[1] > kMaxDrift)) {
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {               // O is complete up to tile i-1 here
                const float down = fast_exp2(m_base[qb] - m_run[qb]);
#pragma unroll
                for (int cb = 0; cb < 8; ++cb) acc[qb][cb] *= down;
                l_run[qb] *= down;
                m_base[qb] = m_run[qb];
                w_cur[qb] = 1.0f;
            }
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // K(i+1): this thread's share landed
        __syncthreads();                 // every wave has finished PV(i-1): the V buffer is free; K(i+1) visible

        // ---- phase 2: P(i) in fp16  |  early QK(i+1)  |  V(i) streams in -----------------------
        // Same stepping.  The exponentials of key block b free that block's score registers, so
        // the MFMA pairs that refill them run one block behind: step (b, ks) carries a quarter of
        // block b's vector work between the two MFMAs of pair ks of block b - 1; the pairs of the
        // last block follow on their own.
        float rs[2] = {0.f, 0.f};
        constexpr int NQK = NB * 4;
        auto k_operand = [&](int j) FPS_INLINE { return ldsK4[j * 64 + lane]; };
        auto qk_pair_half = [&](int j, int qb) FPS_INLINE {
            const int b = j >> 2, ks = j & 3;
            s[qb][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                ring[j & 3].v, qop[qb][ks].v, ks == 0 ? v4f{0.f, 0.f, 0.f, 0.f} : s[qb][b], 0, 0, 0);
        };
        auto phase2_valu = [&](int b, int part) FPS_INLINE {
            const int qb = part >> 1, h = part & 1;
            const float p0 = fast_exp2(__builtin_fmaf(s[qb][b][2 * h], sc, cm[qb]));
            const float p1 = fast_exp2(__builtin_fmaf(s[qb][b][2 * h + 1], sc, cm[qb]));
            rs[qb] += p0;
            rs[qb] += p1;
            uint32_t wd = __builtin_bit_cast(uint32_t, __builtin_convertvector(v2f{p0, p1}, v2h));
            asm volatile("" : "+v"(wd), "+v"(rs[qb]));     // keep the pass in place
            reinterpret_cast<uint32_t*>(&pop[qb][b >> 1].u)[(b & 1) * 2 + h] = wd;
        };
        if (!LAST) {
#pragma unroll
            for (int j = 0; j < 3; ++j) ring[j].u = k_operand(j);
        }
        constexpr int V_STEPS = NB >= 2 ? NB / 2 : 1;      // V's copies are issued in the first half
        constexpr int V_PER_STEP = CPT / V_STEPS;
#pragma unroll
        for (int b = 0; b <= NB; ++b) {
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const int j = (b - 1) * 4 + ks;            // the pair that refills block b - 1
                const bool mfma = !LAST && b >= 1;
                if (mfma) {
                    if (j + 3 < NQK) ring[(j + 3) & 3].u = k_operand(j + 3);
                    qk_pair_half(j, 0);
                }
                if (b < NB) phase2_valu(b, ks);
                if (mfma) qk_pair_half(j, 1);
                if (b < V_STEPS && ks == 0) {
#pragma unroll
                    for (int c = b * V_PER_STEP; c < (b + 1) * V_PER_STEP; ++c) stage_chunk(1, vsrc, c);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            l_run[qb] = __builtin_fmaf(rs[qb], w_cur[qb], l_run[qb]);
            w_prev[qb] = svv * w_cur[qb];
        }
        w0.next();
        w1.next();
        if (!LAST) mask_scores(tile_class(G, w0.vt, w0.vh, w0.vw), w0.js, w0.jb);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // V(i): this thread's share landed
    };
    using T_ = std::true_type;
    using F_ = std::false_type;
    if constexpr (NK == kOneKeyBlock) {
        iteration(T_{}, T_{});
    } else if constexpr (NK == kManyKeyBlocks) {
        iteration(T_{}, F_{});
        for (int it = 1; it + 1 < ntiles; ++it) iteration(F_{}, F_{});
        iteration(F_{}, T_{});
    } else if (ntiles == 1) {
        iteration(T_{}, T_{});
    } else {
        iteration(T_{}, F_{});
        for (int it = 1; it + 1 < ntiles; ++it) iteration(F_{}, F_{});
        iteration(F_{}, T_{});
    }
    // epilogue: the last tile's PV
    __syncthreads();
    {
        v4f tq[2];
#pragma unroll
        for (int cb = 0; cb < 8; ++cb) {
            pv_block(cb, tq);
            pv_accumulate(cb, tq, w_prev);
        }
    }

    float inv[2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        float l = l_run[qb];
        l = sum_over_row_lanes(l);
        inv[qb] = l > 0.f ? 1.0f / l : 0.f;
    }
    __syncthreads();                                       // all waves are done with the staged tiles
    store_rows<BS>(a, bh, u, jq, KBS, tile_class(G, ut, uh, uw), wave, lane, acc, inv,
                   &lds[0][0] + wave * kStoreRegionBytes);
}

// ---------------------------------------------------------------------------------------------
// BF16, 128-slot blocks: v_mfma_f32_32x32x16_bf16 / _f16 (8 passes, twice the work of a 16x16x32)
// and the lane layout of attn_fp8_wide_kernel -- lane (n, h) holds query n, the keys
// 8(r/4) + 4h + r%4 of a 32-key score block and the channels of the same pattern of a 32-channel
// output block.  K and V are single-buffered as in attn_bf16_kernel (two barriers per iteration).
// V's per-tile scale is a power of two here, so the PV product accumulates straight into O: a tile's
// weight 2^E, E = log2(s^V) + m, is applied by keeping O relative to the largest E met so far --
// O is rescaled (exactly) only when that grows, and a tile below it has the difference folded into
// the exponent of its weights before they are rounded to fp16.
// ---------------------------------------------------------------------------------------------
template <bool MB, int NK>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
void attn_bf16_wide_kernel(AttnArgs a, MaskTables) {
    constexpr int BS = 128;
    constexpr int NTHR = 256;
    constexpr int TILE_BYTES = BS * 256;
    constexpr int CPT = (BS * 16) / NTHR;                  // 16-byte chunks per thread per operand tile (8)
    __shared__ __attribute__((aligned(16))) uint8_t lds[2][TILE_BYTES];   // K, V
    const Geom& G = a.g;
    const int KB = MB ? G.KB : 1;
    const int KB_LAST = MB ? G.kb_last : 1;
    const int KBS = MB ? G.KBS : 1;
    const int NS = MB ? G.NS : 1;
    int bh, u, jq;
    if (!work_item(a, KB, &bh, &u, &jq)) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, h = lane >> 5, n = lane & 31;
    const int uw = u % G.nW, uh = (u / G.nW) % G.nH, ut = u / (G.nW * G.nH);
    if (MB && jq >= (ut == G.nT - 1 ? KB_LAST : KB)) {      // a query block of padding only
        zero_block_rows<BS, NTHR>(a, bh, u, jq);
        return;
    }
    const size_t tile0 = (size_t)bh * G.M;
    const uint32_t lds_base = (uint32_t)(uintptr_t)(&lds[0][0]);

    Bf16x8 qop[8];                                         // Q^T, contraction steps of 16 channels
    float m_run = -INFINITY, l_run = 0.f;                  // row reference; sum of 2^14 P relative to it
    float e_ref = 0.f;                                     // the largest weight exponent E met so far
    float alpha_acc = 1.f;                                 // rescale owed to O before the delayed PV
    v16f acc[4];
    {
        const int row = wave * 32 + n;
        const uint4* p = reinterpret_cast<const uint4*>(a.q + (((tile0 + u) * KB + jq) * BS + row) * 256);
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qop[ks].u = p[2 * ks + h];
#pragma unroll
        for (int db = 0; db < 4; ++db) acc[db] = zero16();
    }
    const float sc = kLog2eOverSqrtD;

    TileWalk w0, w1;                                       // tile i and tile i+1
    w0.init(a, KB, KB_LAST, KBS, ut, uh, uw);
    w1 = w0;
    w1.next();
    const int ntiles = w0.n;
    auto tile_of = [&](const TileWalk& w) FPS_INLINE { return (w.vt * G.nH + w.vh) * G.nW + w.vw; };
    const int wave_s = __builtin_amdgcn_readfirstlane(wave);
    auto stage_chunk = [&](int buf, const uint8_t* src, int c) FPS_INLINE {
        dma_chunk_of(c, src + wave_s * (CPT * 1024), lane * 16, lds_base + buf * TILE_BYTES + wave_s * (CPT * 1024));
    };
    auto k_blk = [&](const TileWalk& w) FPS_INLINE { return a.k + ((tile0 + tile_of(w)) * KB + w.jk) * TILE_BYTES; };
    auto v_blk = [&](const TileWalk& w) FPS_INLINE { return a.v + ((tile0 + tile_of(w)) * KB + w.jk) * TILE_BYTES; };
    const uint4* ldsK4 = reinterpret_cast<const uint4*>(lds[0]);
    const uint4* ldsV4 = reinterpret_cast<const uint4*>(lds[1]);

    v16f s[4];                                             // S^T, four blocks of 32 keys
    Bf16x8 pop[8];                                         // P^T in fp16: contraction steps of 16 keys
    Bf16x8 ring[4];                                        // MFMA operands on their way from LDS

    auto mask_scores = [&](int cls, int js, int jb) FPS_INLINE {      // padded keys of a boundary tile: -inf
        cls = __builtin_amdgcn_readfirstlane(cls);
        if (!((a.partial_cls >> cls) & 1u)) return;
        if (!MB) {
#pragma unroll
            for (int kb = 0; kb < 4; ++kb) {
                const uint32_t code = arg_pair_code(cls, kb);
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    s[kb][r] = select_lanes(pair_lane_mask(code, r), s[kb][r], -INFINITY);
            }
        } else {
            uint64_t bm[2];
            block_ballots<BS>(G, cls, js, jb, lane, bm);
            if ((bm[0] & bm[1]) == ~0ull) return;
#pragma unroll
            for (int kb = 0; kb < 4; ++kb) {
                const uint32_t bits = (uint32_t)(bm[kb >> 1] >> (32 * (kb & 1))) >> (4 * h);
#pragma unroll
                for (int r = 0; r < 16; ++r) s[kb][r] = keep_if_bit(s[kb][r], bits, 8 * (r >> 2) + (r & 3));
            }
        }
    };
    // operand j of the K block: key block j/8, contraction step j%8
    auto k_operand = [&](int j) FPS_INLINE { return ldsK4[j * 64 + lane]; };
    auto qk_step = [&](int j) FPS_INLINE {
        const int kb = j >> 3, ks = j & 7;
        s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[j & 3].v, qop[ks].v, ks == 0 ? zero16() : s[kb], 0, 0, 0);
    };
    // PV instructions alternate between two channel blocks, so that consecutive ones do not depend
    // on each other: instruction j -> channel block 2(j/16) + j%2, contraction step (j%16)/2
    auto pv_db = [](int j) { return 2 * (j >> 4) + (j & 1); };
    auto pv_kk = [](int j) { return (j & 15) >> 1; };
    auto v_operand = [&](int j) FPS_INLINE { return ldsV4[(pv_db(j) * 8 + pv_kk(j)) * 64 + lane]; };
    auto pv_step = [&](int j) FPS_INLINE {
        acc[pv_db(j)] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ring[j & 3].h, pop[pv_kk(j)].h, acc[pv_db(j)], 0, 0, 0);
    };

    // prologue: K(0) staged, S(0) computed
#pragma unroll
    for (int c = 0; c < CPT; ++c) stage_chunk(0, k_blk(w0), c);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 32; ++j) {
        ring[j & 3].u = k_operand(j);
        qk_step(j);
    }
    mask_scores(tile_class(G, w0.vt, w0.vh, w0.vw), w0.js, w0.jb);

    auto iteration = [&](auto first_tag, auto last_tag) FPS_INLINE {
        constexpr bool FIRST = decltype(first_tag)::value;
        constexpr bool LAST = decltype(last_tag)::value;
        const int v = tile_of(w0);
        const float svv = load_uniform(a.sv, (tile0 + v) * NS + w0.js);        // 2^e exactly
        const float e_v = (float)((int)((__float_as_uint(svv) >> 23) & 0xFFu) - 127);
        if (a.visited && bh == 0 && tid == 0 && jq == 0 && w0.jk == 0) a.visited[(size_t)u * G.M + v] = 1;
        const uint8_t* ksrc = LAST ? nullptr : k_blk(w1);
        const uint8_t* vsrc = v_blk(w0);
        __syncthreads();                 // every wave has finished QK(i): the K buffer is free; V(i-1) visible

        // ---- phase 1: row maximum of S(i)  |  delayed PV(i-1)  |  K(i+1) streams in ------------
        if (!FIRST && __any(alpha_acc != 1.0f)) {
#pragma unroll
            for (int db = 0; db < 4; ++db) acc[db] *= alpha_acc;
        }
        float mx = __builtin_fmaxf(__builtin_fmaxf(s[0][0], s[0][1]), __builtin_fmaxf(s[0][2], s[0][3]));
        if (!FIRST) {
#pragma unroll
            for (int j = 0; j < 3; ++j) ring[j].u = v_operand(j);
        }
#pragma unroll
        for (int j = 0; j < 32; ++j) {                     // one MFMA and one max3 per step
            if (!FIRST) {
                if (j + 3 < 32) ring[(j + 3) & 3].u = v_operand(j + 3);
                pv_step(j);
            }
            if (j >= 2) {
                mx = __builtin_fmaxf(__builtin_fmaxf(mx, s[j >> 3][2 * (j & 7)]), s[j >> 3][2 * (j & 7) + 1]);
                asm volatile("" : "+v"(mx));
            }
            if (!LAST && (j & 1) == 0 && j < 2 * CPT) stage_chunk(0, ksrc, j >> 1);
            __builtin_amdgcn_sched_barrier(0);
        }
        mx = max_over_row_pair(mx);
        const float m_new = __builtin_fmaxf(m_run, __builtin_ceilf(mx * sc));
        const float alpha_l = fast_exp2(m_run - m_new);    // 0 on the first tile (m_run = -inf)
        m_run = m_new;
        const float e_new = e_v + m_new;
        const float e_top = FIRST ? e_new : __builtin_fmaxf(e_ref, e_new);
        alpha_acc = FIRST ? 1.0f : fast_exp2(e_ref - e_top);
        // <= 0: this tile's weight relative to O's scale; 64 binades down every fp16 weight is zero
        const float below = __builtin_fmaxf(e_new - e_top, -64.0f);
        e_ref = e_top;
        // 2^14 * 2^(S' - m) * 2^below: the factor 2^14 keeps small weights in fp16's normal range and
        // cancels against the row sum, which is taken of the same values
        const float cm = kFp16PScaleLog2 - m_new + below;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // K(i+1): this thread's share landed
        __syncthreads();                 // every wave has finished PV(i-1): the V buffer is free; K(i+1) visible

        // ---- phase 2: P(i) in fp16  |  early QK(i+1)  |  V(i) streams in -----------------------
        // step (kb, ks): a pair of weights of score block kb beside the MFMA (kb - 1, ks) that
        // refills the block whose weights were taken one block earlier
        float rs = 0.f;
        if (!LAST) {
#pragma unroll
            for (int j = 0; j < 3; ++j) ring[j].u = k_operand(j);
        }
#pragma unroll
        for (int kb = 0; kb <= 4; ++kb) {
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                const int j = (kb - 1) * 8 + ks;
                if (!LAST && kb >= 1) {
                    if (j + 3 < 32) ring[(j + 3) & 3].u = k_operand(j + 3);
                    qk_step(j);
                }
                if (kb < 4) {
                    const float p0 = fast_exp2(__builtin_fmaf(s[kb][2 * ks], sc, cm));
                    const float p1 = fast_exp2(__builtin_fmaf(s[kb][2 * ks + 1], sc, cm));
                    rs += p0;
                    rs += p1;
                    uint32_t wd = __builtin_bit_cast(uint32_t, __builtin_convertvector(v2f{p0, p1}, v2h));
                    asm volatile("" : "+v"(wd), "+v"(rs));  // keep the pass in place
                    reinterpret_cast<uint32_t*>(&pop[2 * kb + (ks >> 2)].u)[ks & 3] = wd;
                }
                if (kb * 8 + ks < CPT) stage_chunk(1, vsrc, kb * 8 + ks);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // the row sum was taken of weights scaled by 2^below
        l_run = __builtin_fmaf(rs, fast_exp2(-below), l_run * alpha_l);
        w0.next();
        w1.next();
        if (!LAST) mask_scores(tile_class(G, w0.vt, w0.vh, w0.vw), w0.js, w0.jb);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // V(i): this thread's share landed
    };
    using T_ = std::true_type;
    using F_ = std::false_type;
    if constexpr (NK == kOneKeyBlock) {
        iteration(T_{}, T_{});
    } else if constexpr (NK == kManyKeyBlocks) {
        iteration(T_{}, F_{});
        for (int it = 1; it + 1 < ntiles; ++it) iteration(F_{}, F_{});
        iteration(F_{}, T_{});
    } else if (ntiles == 1) {
        iteration(T_{}, T_{});
    } else {
        iteration(T_{}, F_{});
        for (int it = 1; it + 1 < ntiles; ++it) iteration(F_{}, F_{});
        iteration(F_{}, T_{});
    }
    // epilogue: the last tile's PV
    __syncthreads();
    if (__any(alpha_acc != 1.0f)) {
#pragma unroll
        for (int db = 0; db < 4; ++db) acc[db] *= alpha_acc;
    }
#pragma unroll
    for (int j = 0; j < 32; ++j) {
        ring[j & 3].u = v_operand(j);
        pv_step(j);
    }
    const float l = sum_over_row_pair(l_run);
    const float inv = l > 0.f ? fast_exp2(e_ref - m_run) / l : 0.f;
    __syncthreads();                                       // all waves are done with the staged tiles
    store_rows_wide(a, bh, u, jq, KBS, tile_class(G, ut, uh, uw), wave, lane, acc, inv,
                    &lds[0][0] + wave * kStoreRegionBytes);
}

// Debug: raw E4M3 score accumulators sum_c q_ic * k_jc of one tile pair, produced by the same MFMA
// instruction and operand layouts as attn_fp8_kernel; out[i*BS + j], query-major.
template <int BS>
__global__ __launch_bounds__(BS * 2) void scores_fp8_kernel(const uint8_t* __restrict__ q_tile,
                                                            const uint8_t* __restrict__ k_tile,
                                                            float* __restrict__ out_tile, int out_pitch) {
    constexpr int NB = BS / 16;
    // workgroup (x, y) = (key block, query block) of the tile pair
    const uint8_t* q = q_tile + (size_t)blockIdx.y * BS * 128;
    const uint8_t* k = k_tile + (size_t)blockIdx.x * BS * 128;
    float* out = out_tile + (size_t)blockIdx.y * BS * out_pitch + (size_t)blockIdx.x * BS;
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
            for (int r = 0; r < 4; ++r) out[(size_t)row * out_pitch + 16 * b + 4 * g + r] = s[r];
        }
    }
}

// The same for 128-slot blocks: the 32x32x64 instruction and operand layouts of attn_fp8_wide_kernel.
__global__ __launch_bounds__(256) void scores_fp8_wide_kernel(const uint8_t* __restrict__ q_tile,
                                                              const uint8_t* __restrict__ k_tile,
                                                              float* __restrict__ out_tile, int out_pitch) {
    const uint8_t* q = q_tile + (size_t)blockIdx.y * 128 * 128;
    const uint8_t* k = k_tile + (size_t)blockIdx.x * 128 * 128;
    float* out = out_tile + (size_t)blockIdx.y * 128 * out_pitch + (size_t)blockIdx.x * 128;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, h = lane >> 5, n = lane & 31;
    const uint4* k4 = reinterpret_cast<const uint4*>(k);
    const int row = wave * 32 + n;
    const uint4* p = reinterpret_cast<const uint4*>(q + row * 128 + 32 * h);
    const v8i qop[2] = {make_v8i(p[0], p[1]), make_v8i(p[4], p[5])};
    for (int kb = 0; kb < 4; ++kb) {
        v16f s = zero16();
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            const v8i kop = make_v8i(k4[((kb * 2 + ks) * 2 + 0) * 64 + lane], k4[((kb * 2 + ks) * 2 + 1) * 64 + lane]);
            s = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(kop, qop[ks], s, 0, 0, 0, 0, 0, 0);
        }
#pragma unroll
        for (int r = 0; r < 16; ++r)
            out[(size_t)row * out_pitch + 32 * kb + 8 * (r >> 2) + 4 * h + (r & 3)] = s[r];
    }
}

// MFMA-only loop: 8 independent accumulator chains of the attention kernel's matrix instruction.
__global__ __launch_bounds__(256) void mfma_rate_kernel(float* __restrict__ sink, int iters, int x) {
    v8i a = {x, x, x, x, x, x, x, x};
    v8i b = a;
    v4f c[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) c[i] = v4f{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
            c[i] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, c[i], 0, 0, 0, 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) s += c[i][0] + c[i][1] + c[i][2] + c[i][3];
    sink[blockIdx.x * 256 + threadIdx.x] = s;
}

int launch_mfma_rate(int workgroups, int iters, float* sink, hipStream_t st) {
    mfma_rate_kernel<<<workgroups, 256, 0, st>>>(sink, iters, 0x38383838);   // E4M3 code of 1.0 in every byte
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? FPS_OK : hip_fail(e, "mfma rate launch");
}

int launch_scores_fp8(const Geom& g, const void* q, const void* k, int bh, int u, int v, float* out,
                      hipStream_t st) {
    // every (query block, key block) pair of the tile pair; out is [TSP][TSP], query-major
    const size_t tile_bytes = (size_t)g.TSP * 128;
    const uint8_t* qp = (const uint8_t*)q + ((size_t)bh * g.M + u) * tile_bytes;
    const uint8_t* kp = (const uint8_t*)k + ((size_t)bh * g.M + v) * tile_bytes;
    const dim3 grid(g.KB, g.KB);
    if (g.BS == 128) scores_fp8_wide_kernel<<<grid, 256, 0, st>>>(qp, kp, out, g.TSP);
    else             scores_fp8_kernel<32><<<grid, 64, 0, st>>>(qp, kp, out, g.TSP);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? FPS_OK : hip_fail(e, "debug scores launch");
}

int launch_scores_block_fp8(const Geom& g, const void* q, const void* k, int bh, int u, int jq, int v,
                            int jk, float* out, hipStream_t st) {
    const size_t blk_bytes = (size_t)g.BS * 128;
    const uint8_t* qp = (const uint8_t*)q + (((size_t)bh * g.M + u) * g.KB + jq) * blk_bytes;
    const uint8_t* kp = (const uint8_t*)k + (((size_t)bh * g.M + v) * g.KB + jk) * blk_bytes;
    if (g.BS == 128) scores_fp8_wide_kernel<<<dim3(1, 1), 256, 0, st>>>(qp, kp, out, g.BS);
    else             scores_fp8_kernel<32><<<dim3(1, 1), 64, 0, st>>>(qp, kp, out, g.BS);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? FPS_OK : hip_fail(e, "debug block scores launch");
}

int launch_attn(const Geom& g, const fps_window& win, int prec, const void* q, const void* k,
                const void* v, const float* sq, const float* sk, const float* sv, int vscale,
                void* out, int out_f32, int out_raster, uint8_t* visited, hipStream_t st) {
    AttnArgs a;
    a.q = (const uint8_t*)q; a.k = (const uint8_t*)k; a.v = (const uint8_t*)v;
    a.sq = sq; a.sk = sk; a.sv = sv;
    a.out = out; a.visited = visited;
    a.g = g;
    a.rt = win.wt / 2; a.rh = win.wh / 2; a.rw = win.ww / 2;
    a.edge_shift = win.edge == FPS_EDGE_SHIFT;
    a.out_f32 = out_f32;
    a.out_raster = out_raster;
    a.total = g.BH * g.M * g.KB;
    a.chunk = (a.total + 7) / 8;
    a.partial_cls = 0;
    for (int c = 0; c < 8; ++c)
        if (g.TS != g.TSP || ((c & 4) && g.lastT < g.Tt) || ((c & 2) && g.lastH < g.Th) ||
            ((c & 1) && g.lastW < g.Tw))
            a.partial_cls |= 1u << c;
    MaskTables t;
    memset(&t, 0, sizeof(t));
    if (g.KB == 1) {
        for (int c = 0; c < 8; ++c) {
            bool ok[128];
            for (int r = 0; r < 128; ++r) ok[r] = r < g.BS && slot_is_token(g, c, r);
            for (int i = 0; i < 32; ++i) {
                uint64_t m = 0;
                const int b = i >> 2, r = i & 3;
                for (int lane = 0; lane < 64; ++lane)
                    if (ok[16 * b + 4 * (lane >> 4) + r]) m |= 1ull << lane;
                t.lane_mask[c][i] = m;
            }
            for (int kb = 0; kb < 4; ++kb)
                for (int r = 0; r < 16; ++r)
                    for (int h = 0; h < 2; ++h)
                        if (ok[32 * kb + 8 * (r >> 2) + 4 * h + (r & 3)]) t.pair_code[c][kb] |= 1u << (2 * r + h);
        }
    }
    const int grid = a.chunk * 8;
    const bool multi = g.KB > 1;
    const bool vch = vscale == FPS_VSCALE_CHANNEL;
    // one-block tiles: every work item walks as many key blocks as its window has tiles, and a corner
    // tile of the grid has the fewest -- one exactly when no axis has both a radius and a neighbour
    const int corner = (a.rt < g.nT ? a.rt + 1 : g.nT) * (a.rh < g.nH ? a.rh + 1 : g.nH) *
                       (a.rw < g.nW ? a.rw + 1 : g.nW);
    const bool one = corner == 1;
    // tiles of several blocks: a lower bound on the key blocks of any item
    const bool many = (long long)corner * (g.KB < g.kb_last ? g.KB : g.kb_last) >= 2;
#define FPS_LAUNCH_FP8(KERNEL_, THREADS_)                                                          \
    do {                                                                                           \
        if (multi && many) {                                                                       \
            if (vch) KERNEL_(true, true, kManyKeyBlocks)<<<grid, THREADS_, 0, st>>>(a, t);         \
            else     KERNEL_(false, true, kManyKeyBlocks)<<<grid, THREADS_, 0, st>>>(a, t);        \
        } else if (multi) {                                                                        \
            if (vch) KERNEL_(true, true, kAnyKeyBlocks)<<<grid, THREADS_, 0, st>>>(a, t);          \
            else     KERNEL_(false, true, kAnyKeyBlocks)<<<grid, THREADS_, 0, st>>>(a, t);         \
        } else if (one) {                                                                          \
            if (vch) KERNEL_(true, false, kOneKeyBlock)<<<grid, THREADS_, 0, st>>>(a, t);          \
            else     KERNEL_(false, false, kOneKeyBlock)<<<grid, THREADS_, 0, st>>>(a, t);         \
        } else {                                                                                   \
            if (vch) KERNEL_(true, false, kManyKeyBlocks)<<<grid, THREADS_, 0, st>>>(a, t);        \
            else     KERNEL_(false, false, kManyKeyBlocks)<<<grid, THREADS_, 0, st>>>(a, t);       \
        }                                                                                          \
    } while (0)
#define FPS_FP8_WIDE(VCH_, MB_, NK_) attn_fp8_wide_kernel<VCH_, MB_, NK_>
#define FPS_FP8_SMALL(VCH_, MB_, NK_) attn_fp8_kernel<32, VCH_, MB_, NK_>
#define FPS_LAUNCH_BF16(KERNEL_, THREADS_)                                                         \
    do {                                                                                           \
        if (multi && many) KERNEL_(true, kManyKeyBlocks)<<<grid, THREADS_, 0, st>>>(a, t);         \
        else if (multi) KERNEL_(true, kAnyKeyBlocks)<<<grid, THREADS_, 0, st>>>(a, t);             \
        else if (one) KERNEL_(false, kOneKeyBlock)<<<grid, THREADS_, 0, st>>>(a, t);               \
        else          KERNEL_(false, kManyKeyBlocks)<<<grid, THREADS_, 0, st>>>(a, t);             \
    } while (0)
#define FPS_BF16_WIDE(MB_, NK_) attn_bf16_wide_kernel<MB_, NK_>
#define FPS_BF16_SMALL(MB_, NK_) attn_bf16_kernel<32, MB_, NK_>
    if (prec == FPS_PREC_FP8) {
        if (g.BS == 128) FPS_LAUNCH_FP8(FPS_FP8_WIDE, 256); else FPS_LAUNCH_FP8(FPS_FP8_SMALL, 64);
    } else {
        if (g.BS == 128) FPS_LAUNCH_BF16(FPS_BF16_WIDE, 256); else FPS_LAUNCH_BF16(FPS_BF16_SMALL, 64);
    }
#undef FPS_LAUNCH_FP8
#undef FPS_FP8_WIDE
#undef FPS_FP8_SMALL
#undef FPS_LAUNCH_BF16
#undef FPS_BF16_WIDE
#undef FPS_BF16_SMALL
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? FPS_OK : hip_fail(e, "attention launch");
}

}  // namespace fps
