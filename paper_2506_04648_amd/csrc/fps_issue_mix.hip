// Debug: how matrix and vector instructions share a SIMD's issue port.  A loop of groups, each one
// matrix instruction followed by NV independent vector instructions, timed with the shader clock
// inside the kernel; no memory traffic in the loop.  The attention kernels are bounded by exactly
// this mix (Sec. 3.4 states the kernel as tensor-core bound; on this chip the softmax's vector work
// beside each MFMA decides), so the table this kernel produces is the yardstick their measured
// cycles per key block are compared with.
#include "fps_internal.h"

namespace fps {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

enum { kMixFp8 = 0, kMixBf16 = 1, kMixNone = 2, kMixFp8Wide = 3, kMixBf16Wide = 4 };
typedef float v16f __attribute__((ext_vector_type(16)));
enum { kOpFma = 0, kOpExp = 1 };

// KIND: the matrix instruction (v_mfma_f32_16x16x128_f8f6f4 with E4M3 operands, 8 passes;
// v_mfma_f32_16x16x32_bf16, 4 passes; none; v_mfma_f32_32x32x64_f8f6f4, 16 passes and twice the
// work of the first; or v_mfma_f32_32x32x16_bf16, 8 passes and twice the work of the second).  NV v_fma_f32 per group.  Eight accumulator chains,
// so a matrix instruction depends on the one issued eight groups earlier; every vector instruction
// continues its own chain, one per group.  cycles[workgroup * 4 + wave] receives the wave's shader
// clocks for the whole loop.
template <int KIND, int NV>
__global__ __launch_bounds__(256) void issue_mix_kernel(float* __restrict__ sink,
                                                        unsigned long long* __restrict__ cycles,
                                                        int iters, int x) {
    extern __shared__ uint8_t residency_limit[];            // sized by the host to fix workgroups per CU
    v8i a8 = {x, x, x, x, x, x, x, x};
    v8i b8 = a8;
    const v8bf a16 = __builtin_bit_cast(v8bf, (int __attribute__((ext_vector_type(4)))){x, x, x, x});
    const v8bf b16 = a16;
    v4f c[8];
    v16f cw[4];                                             // the 32x32 shape: four chains of 16 registers
#pragma unroll
    for (int i = 0; i < 8; ++i) c[i] = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) cw[i][r] = 0.f;
    constexpr int NF = NV > 0 ? NV : 1;
    float f[NF];
#pragma unroll
    for (int j = 0; j < NF; ++j) f[j] = 0.25f + 0.001f * (float)(threadIdx.x + j);
    const float k1 = 0.999f + 1e-13f * (float)x, k2 = 1e-4f;   // not a compile-time constant; the chains stay bounded
    const unsigned long long t0 = __builtin_readcyclecounter();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (KIND == kMixFp8)
                c[i] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a8, b8, c[i], 0, 0, 0, 0, 0, 0);
            else if (KIND == kMixBf16)
                c[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a16, b16, c[i], 0, 0, 0);
            else if (KIND == kMixFp8Wide)
                cw[i & 3] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a8, b8, cw[i & 3], 0, 0, 0, 0, 0, 0);
            else if (KIND == kMixBf16Wide)
                cw[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a16, b16, cw[i & 3], 0, 0, 0);
#pragma unroll
            for (int j = 0; j < NV; ++j) f[j] = __builtin_fmaf(f[j], k1, k2);
            __builtin_amdgcn_sched_barrier(0);              // groups stay as written
        }
    }
    const unsigned long long t1 = __builtin_readcyclecounter();
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) s += c[i][0] + c[i][1] + c[i][2] + c[i][3];
#pragma unroll
    for (int i = 0; i < 4; ++i) s += cw[i][0] + cw[i][5] + cw[i][10] + cw[i][15];
#pragma unroll
    for (int j = 0; j < NF; ++j) s += f[j];
    sink[blockIdx.x * 256 + threadIdx.x] = s;
    if ((threadIdx.x & 63) == 0) cycles[blockIdx.x * 4 + (threadIdx.x >> 6)] = t1 - t0;
    (void)residency_limit;
}

// The same with the transcendental unit: NV times per group f <- exp2(f) - 1, which keeps f in
// (-1, 0): one v_exp_f32 and one v_add_f32 each.
template <int KIND, int NV>
__global__ __launch_bounds__(256) void issue_mix_exp_kernel(float* __restrict__ sink,
                                                            unsigned long long* __restrict__ cycles,
                                                            int iters, int x) {
    extern __shared__ uint8_t residency_limit[];
    v8i a8 = {x, x, x, x, x, x, x, x};
    v8i b8 = a8;
    const v8bf a16 = __builtin_bit_cast(v8bf, (int __attribute__((ext_vector_type(4)))){x, x, x, x});
    const v8bf b16 = a16;
    v4f c[8];
    v16f cw[4];                                             // the 32x32 shape: four chains of 16 registers
#pragma unroll
    for (int i = 0; i < 8; ++i) c[i] = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) cw[i][r] = 0.f;
    constexpr int NF = NV > 0 ? NV : 1;
    float f[NF];
#pragma unroll
    for (int j = 0; j < NF; ++j) f[j] = -0.5f - 0.001f * (float)((threadIdx.x + j) & 63);
    const unsigned long long t0 = __builtin_readcyclecounter();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (KIND == kMixFp8)
                c[i] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a8, b8, c[i], 0, 0, 0, 0, 0, 0);
            else if (KIND == kMixBf16)
                c[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a16, b16, c[i], 0, 0, 0);
            else if (KIND == kMixFp8Wide)
                cw[i & 3] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a8, b8, cw[i & 3], 0, 0, 0, 0, 0, 0);
            else if (KIND == kMixBf16Wide)
                cw[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a16, b16, cw[i & 3], 0, 0, 0);
#pragma unroll
            for (int j = 0; j < NV; ++j) f[j] = __builtin_amdgcn_exp2f(f[j]) - 1.0f;   // stays in (-1, 0)
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    const unsigned long long t1 = __builtin_readcyclecounter();
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) s += c[i][0] + c[i][1] + c[i][2] + c[i][3];
#pragma unroll
    for (int i = 0; i < 4; ++i) s += cw[i][0] + cw[i][5] + cw[i][10] + cw[i][15];
#pragma unroll
    for (int j = 0; j < NF; ++j) s += f[j];
    sink[blockIdx.x * 256 + threadIdx.x] = s;
    if ((threadIdx.x & 63) == 0) cycles[blockIdx.x * 4 + (threadIdx.x >> 6)] = t1 - t0;
    (void)residency_limit;
}

template <int KIND, int NV>
static hipError_t launch_one(int op, int workgroups, size_t lds, int iters, float* sink,
                             unsigned long long* cycles, hipStream_t st) {
    const int x = 0x38383838;                               // E4M3 1.0 in every byte; a small bf16 as halves
    if (op == kOpFma) {
        auto kern = issue_mix_kernel<KIND, NV>;
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        kern<<<workgroups, 256, lds, st>>>(sink, cycles, iters, x);
    } else {
        auto kern = issue_mix_exp_kernel<KIND, NV>;
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        kern<<<workgroups, 256, lds, st>>>(sink, cycles, iters, x);
    }
    return hipGetLastError();
}

template <int KIND>
static hipError_t launch_kind(int nv, int op, int workgroups, size_t lds, int iters, float* sink,
                              unsigned long long* cycles, hipStream_t st, bool* known) {
    *known = true;
    switch (nv) {
        case 0: return launch_one<KIND, 0>(op, workgroups, lds, iters, sink, cycles, st);
        case 1: return launch_one<KIND, 1>(op, workgroups, lds, iters, sink, cycles, st);
        case 2: return launch_one<KIND, 2>(op, workgroups, lds, iters, sink, cycles, st);
        case 3: return launch_one<KIND, 3>(op, workgroups, lds, iters, sink, cycles, st);
        case 4: return launch_one<KIND, 4>(op, workgroups, lds, iters, sink, cycles, st);
        case 6: return launch_one<KIND, 6>(op, workgroups, lds, iters, sink, cycles, st);
        case 8: return launch_one<KIND, 8>(op, workgroups, lds, iters, sink, cycles, st);
        case 12: return launch_one<KIND, 12>(op, workgroups, lds, iters, sink, cycles, st);
        case 16: return launch_one<KIND, 16>(op, workgroups, lds, iters, sink, cycles, st);
        case 24: return launch_one<KIND, 24>(op, workgroups, lds, iters, sink, cycles, st);
        case 32: return launch_one<KIND, 32>(op, workgroups, lds, iters, sink, cycles, st);
        default: *known = false; return hipSuccess;
    }
}

int launch_issue_mix(int kind, int nv, int op, int workgroups_per_cu, int workgroups, int iters,
                     float* sink, unsigned long long* cycles, hipStream_t st) {
    // a workgroup asks for a little less than 1/n of the CU's 160 KB of LDS (n exact shares do not
    // all fit), so n of them are resident per CU and no more: n waves per SIMD (a workgroup is four
    // waves, one per SIMD)
    size_t lds = (size_t)(160 * 1024) / (size_t)workgroups_per_cu - 1024;
    if (workgroups_per_cu == 2) lds = 64 * 1024;           // two of 64 KB fit, a third does not
    bool known = false;
    hipError_t e;
    if (kind == kMixFp8)       e = launch_kind<kMixFp8>(nv, op, workgroups, lds, iters, sink, cycles, st, &known);
    else if (kind == kMixBf16) e = launch_kind<kMixBf16>(nv, op, workgroups, lds, iters, sink, cycles, st, &known);
    else if (kind == kMixFp8Wide) e = launch_kind<kMixFp8Wide>(nv, op, workgroups, lds, iters, sink, cycles, st, &known);
    else if (kind == kMixBf16Wide) e = launch_kind<kMixBf16Wide>(nv, op, workgroups, lds, iters, sink, cycles, st, &known);
    else                       e = launch_kind<kMixNone>(nv, op, workgroups, lds, iters, sink, cycles, st, &known);
    if (!known) {
        set_error("valu_per_mfma must be one of 0 1 2 3 4 6 8 12 16 24 32");
        return FPS_ERR_INVALID_ARG;
    }
    return e == hipSuccess ? FPS_OK : hip_fail(e, "issue mix launch");
}

}  // namespace fps
