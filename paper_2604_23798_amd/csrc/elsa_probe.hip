// Measurement hook, not part of the attention path: what single instruction kinds cost to issue on gfx950, alone
// and beside the matrix-core instructions of another wave of the same SIMD.  The fold between the two MFMA
// contractions is made of these kinds (exponentials, FMAs, adds, maxima, FP16 conversions), so their issue cost
// -- and whether it hides behind another wave's MFMAs -- is what separates the kernels from the matrix-core roof.
//
// One block per CU, 256 or 512 threads (one or two waves per SIMD).  Waves 0-3 run kind_a, waves 4-7 kind_b:
// `iters` iterations of 16 independent instructions of the kind (8 for the MFMA kinds).  Every wave of block 0
// reports the time it took in ticks of the constant 100 MHz counter: out[wave], 8 floats.
#include "elsa_common.hpp"

namespace elsa {

namespace {

enum { P_EXP = 0, P_FMA, P_ADD, P_MAX3, P_CVT_PK_F16, P_MFMA_F32, P_MFMA_F16, P_NONE, P_KINDS };

template <int KIND>
__device__ __forceinline__ void issue16(float (&x)[8], unsigned (&h)[8], f32x16 (&acc)[4], f16x8 ha, f16x8 hb, float a, float b) {
#pragma unroll
    for (int r = 0; r < 2; ++r)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if constexpr (KIND == P_EXP) asm volatile("v_exp_f32 %0, %0" : "+v"(x[i]));
            else if constexpr (KIND == P_FMA) asm volatile("v_fma_f32 %0, %1, %2, %0" : "+v"(x[i]) : "v"(a), "v"(b));
            else if constexpr (KIND == P_ADD) asm volatile("v_add_f32 %0, %1, %0" : "+v"(x[i]) : "v"(a));
            else if constexpr (KIND == P_MAX3) asm volatile("v_max3_f32 %0, %0, %1, %2" : "+v"(x[i]) : "v"(a), "v"(b));
            else if constexpr (KIND == P_CVT_PK_F16) asm volatile("v_cvt_pk_f16_f32 %0, %1, %2" : "=v"(h[i]) : "v"(x[i]), "v"(x[(i + 1) & 7]));
            else if constexpr (KIND == P_MFMA_F32) {
                if (i < 4) asm volatile("v_mfma_f32_32x32x2_f32 %0, %1, %2, %0" : "+v"(acc[i]) : "v"(a), "v"(b));
            } else if constexpr (KIND == P_MFMA_F16) {
                if (i < 4) asm volatile("v_mfma_f32_32x32x16_f16 %0, %1, %2, %0" : "+v"(acc[i]) : "v"(ha), "v"(hb));
            }
        }
}

template <int KIND>
__device__ __forceinline__ void run_kind(int iters, float (&x)[8], unsigned (&h)[8], f32x16 (&acc)[4], f16x8 ha, f16x8 hb, float a, float b) {
    for (int it = 0; it < iters; ++it) issue16<KIND>(x, h, acc, ha, hb, a, b);
}

__device__ __forceinline__ void dispatch(int kind, int iters, float (&x)[8], unsigned (&h)[8], f32x16 (&acc)[4], f16x8 ha, f16x8 hb, float a, float b) {
    switch (kind) {
        case P_EXP: run_kind<P_EXP>(iters, x, h, acc, ha, hb, a, b); break;
        case P_FMA: run_kind<P_FMA>(iters, x, h, acc, ha, hb, a, b); break;
        case P_ADD: run_kind<P_ADD>(iters, x, h, acc, ha, hb, a, b); break;
        case P_MAX3: run_kind<P_MAX3>(iters, x, h, acc, ha, hb, a, b); break;
        case P_CVT_PK_F16: run_kind<P_CVT_PK_F16>(iters, x, h, acc, ha, hb, a, b); break;
        case P_MFMA_F32: run_kind<P_MFMA_F32>(iters, x, h, acc, ha, hb, a, b); break;
        case P_MFMA_F16: run_kind<P_MFMA_F16>(iters, x, h, acc, ha, hb, a, b); break;
        default: break;
    }
}

__global__ __launch_bounds__(512) void issue_probe_kernel(float *out, float *sink, int kind_a, int kind_b, int iters, float a, float b) {
    f32x16 acc[4];
    for (int c = 0; c < 4; ++c)
        for (int i = 0; i < 16; ++i) acc[c][i] = 0.f;
    f16x8 ha, hb;
    for (int i = 0; i < 8; ++i) {
        ha[i] = (_Float16)(a * i);
        hb[i] = (_Float16)(b * i);
    }
    float x[8];
    unsigned h[8];
    for (int i = 0; i < 8; ++i) {
        x[i] = -0.001f * (threadIdx.x + i);
        h[i] = 0x3c003800u + i;
    }
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const unsigned long long t0 = wall_clock64();
    dispatch(wave < 4 ? kind_a : kind_b, iters, x, h, acc, ha, hb, a, b);     // wave-uniform
    const unsigned long long t1 = wall_clock64();
    float s = 0.f;
    for (int c = 0; c < 4; ++c)
        for (int i = 0; i < 16; ++i) s += acc[c][i];
    for (int i = 0; i < 8; ++i) s += x[i] + (float)h[i];
    sink[blockIdx.x * blockDim.x + threadIdx.x] = s;                          // keeps the instruction streams alive
    if (blockIdx.x == 0 && (threadIdx.x & 63) == 0) out[wave] = (float)(t1 - t0);
}

}  // namespace

// out: 8 floats (ticks per wave of block 0) followed by the sink of kNumCu * 512 floats.
int launch_issue_probe(float *out, int kind_a, int kind_b, int waves_per_simd, int iters, hipStream_t s) {
    if (kind_a < 0 || kind_a >= P_KINDS || kind_b < 0 || kind_b >= P_KINDS) return (int)hipErrorInvalidValue;
    if ((waves_per_simd != 1 && waves_per_simd != 2) || iters < 1 || iters > (1 << 20)) return (int)hipErrorInvalidValue;
    hipLaunchKernelGGL(issue_probe_kernel, dim3(kNumCu), dim3(256 * waves_per_simd), 0, s, out, out + 8, kind_a, kind_b, iters, 1e-3f, 1e-3f);
    return (int)hipGetLastError();
}

}  // namespace elsa
