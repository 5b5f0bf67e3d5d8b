// Measurement hook, not part of the attention path: what single instruction kinds cost to issue on gfx950, alone
// and beside the matrix-core instructions of another wave of the same SIMD.  The fold between the two MFMA
// contractions is made of these kinds (exponentials, FMAs, adds, maxima, FP16 conversions), so their issue cost
// -- and whether it hides behind another wave's MFMAs -- is what separates the kernels from the matrix-core roof.
//
// One block per CU, 256 or 512 threads (one or two waves per SIMD).  Waves 0-3 run kind_a, waves 4-7 kind_b:
// `iters` iterations of 16 independent instructions of the kind (8 for the MFMA kinds).  Every wave of block 0
// reports the time it took in ticks of the constant 100 MHz counter: out[wave], 8 floats.
//
// Kinds 8-10 are a register-only model of one fold step of the FP16 256-row tile (two query groups of 32 rows x 32 keys
// per wave, d = 64, reference not renewed): per iteration 2 x 4 score MFMAs, 2 x (16 FMA + 16 exponentials + 16 additions
// + 8 conversions + the limit test), 2 x 4 PV MFMAs, on constant fragments -- no LDS, no staging, no barrier.  8 = the
// MFMAs alone, 9 = the fold alone, 10 = the whole step.  What the real kernel takes beyond kind 10 is the cost of moving
// its tiles.
#include "elsa_common.hpp"

namespace elsa {

namespace {

enum { P_EXP = 0, P_FMA, P_ADD, P_MAX3, P_CVT_PK_F16, P_MFMA_F32, P_MFMA_F16, P_NONE, P_STEP_MFMA, P_STEP_FOLD, P_STEP_WHOLE, P_KINDS };

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

// MODE bit 0: score MFMAs, bit 1: fold, bit 2: PV MFMAs
template <int MODE>
__device__ __forceinline__ float step_model(int iters, float c, float a) {
    constexpr int NQ = 2;
    f16x8 kf[4], qf[NQ][4];
    for (int k = 0; k < 4; ++k)
        for (int i = 0; i < 8; ++i) {
            kf[k][i] = (_Float16)(a * (float)((threadIdx.x + i + k) & 15));
            for (int g = 0; g < NQ; ++g) qf[g][k][i] = (_Float16)(a * (float)((threadIdx.x * 5 + i + k + g) & 15));
        }
    f32x16 o[NQ][2];
    float S[NQ], nmc[NQ];
    f16x8 p[NQ][2];
    for (int g = 0; g < NQ; ++g) {
        S[g] = 0.f;
        nmc[g] = -a;
        for (int i = 0; i < 16; ++i) { o[g][0][i] = 0.f; o[g][1][i] = 0.f; }
        for (int i = 0; i < 8; ++i) { p[g][0][i] = (_Float16)a; p[g][1][i] = (_Float16)a; }
    }
    for (int it = 0; it < iters; ++it) {
        f32x16 s[NQ];
#pragma unroll
        for (int g = 0; g < NQ; ++g) {
            for (int i = 0; i < 16; ++i) s[g][i] = 0.f;
            if constexpr ((MODE & 1) != 0) {
#pragma unroll
                for (int k = 0; k < 4; ++k) s[g] = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf[k], qf[g][k], s[g], 0, 0, 0);
            } else {
                for (int i = 0; i < 16; ++i) s[g][i] = (float)p[g][i >> 3][i & 7];
            }
        }
#pragma unroll
        for (int g = 0; g < NQ; ++g) {
            if constexpr ((MODE & 2) != 0) {
                float e[16];
#pragma unroll
                for (int i = 0; i < 16; ++i) e[i] = exp2_fast(__builtin_fmaf(s[g][i], c, nmc[g]));
                float ps = e[0];
#pragma unroll
                for (int i = 1; i < 16; ++i) ps += e[i];
                if (__builtin_amdgcn_ballot_w64(!(ps < 1024.f)) != 0) { nmc[g] -= 1.f; S[g] *= 0.5f; }   // (not taken on these operands)
                S[g] += ps;
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    p[g][i >> 2][2 * (i & 3)] = (_Float16)e[2 * i];
                    p[g][i >> 2][2 * (i & 3) + 1] = (_Float16)e[2 * i + 1];
                }
            } else {
                S[g] += s[g][0];
            }
        }
#pragma unroll
        for (int g = 0; g < NQ; ++g) {
            if constexpr ((MODE & 4) != 0) {
#pragma unroll
                for (int kk = 0; kk < 2; ++kk) {
                    o[g][0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf[kk], p[g][kk], o[g][0], 0, 0, 0);
                    o[g][1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf[2 + kk], p[g][kk], o[g][1], 0, 0, 0);
                }
            }
        }
    }
    float r = 0.f;
    for (int g = 0; g < NQ; ++g) {
        r += S[g] + nmc[g];
        for (int i = 0; i < 16; ++i) r += o[g][0][i] + o[g][1][i];
        for (int i = 0; i < 8; ++i) r += (float)p[g][0][i] + (float)p[g][1][i];
    }
    return r;
}

// Same reporting as the issue probe: waves 0-3 run mode_a, waves 4-7 mode_b (0 = nothing).
__global__ __launch_bounds__(512, 1) void step_model_kernel(float *out, float *sink, int mode_a, int mode_b, int iters, float c, float a) {
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int mode = wave < 4 ? mode_a : mode_b;                              // wave-uniform
    const unsigned long long t0 = wall_clock64();
    float r = 0.f;
    if (mode == 5) r = step_model<5>(iters, c, a);
    else if (mode == 2) r = step_model<2>(iters, c, a);
    else if (mode == 7) r = step_model<7>(iters, c, a);
    const unsigned long long t1 = wall_clock64();
    sink[blockIdx.x * blockDim.x + threadIdx.x] = r;
    if (blockIdx.x == 0 && (threadIdx.x & 63) == 0) out[wave] = (float)(t1 - t0);
}

}  // namespace

// out: 8 floats (ticks per wave of block 0) followed by the sink of kNumCu * 512 floats.
int launch_issue_probe(float *out, int kind_a, int kind_b, int waves_per_simd, int iters, hipStream_t s) {
    if (kind_a < 0 || kind_a >= P_KINDS || kind_b < 0 || kind_b >= P_KINDS) return (int)hipErrorInvalidValue;
    if ((waves_per_simd != 1 && waves_per_simd != 2) || iters < 1 || iters > (1 << 20)) return (int)hipErrorInvalidValue;
    const bool model_a = kind_a >= P_STEP_MFMA, model_b = kind_b >= P_STEP_MFMA;
    if (model_a || model_b) {
        // the step model runs beside itself or beside nothing
        if ((!model_a && kind_a != P_NONE) || (!model_b && kind_b != P_NONE)) return (int)hipErrorInvalidValue;
        static const int modes[3] = {5, 2, 7};
        const int ma = model_a ? modes[kind_a - P_STEP_MFMA] : 0, mb = model_b ? modes[kind_b - P_STEP_MFMA] : 0;
        hipLaunchKernelGGL(step_model_kernel, dim3(kNumCu), dim3(256 * waves_per_simd), 0, s, out, out + 8, ma, mb, iters, 0.18f, 1e-2f);
        return (int)hipGetLastError();
    }
    hipLaunchKernelGGL(issue_probe_kernel, dim3(kNumCu), dim3(256 * waves_per_simd), 0, s, out, out + 8, kind_a, kind_b, iters, 1e-3f, 1e-3f);
    return (int)hipGetLastError();
}

}  // namespace elsa
