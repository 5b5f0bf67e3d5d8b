// ELSA forward for many small independent problems (window attention: n of a few dozen to a few
// hundred tokens, thousands of (window, head) pairs), FP32 MFMA, no LDS.
//
// One wave owns 32*NQ query rows of one (batch, head) and walks its keys 32 at a time; nothing is
// shared between waves, so K and V fragments go straight from memory (L2 / L1) into the MFMA
// operand registers through buffer descriptors -- no staging, no barrier, and the occupancy is set
// by registers alone.  The fold of the tile into (m, S, W) is the one of the tiled kernel: scores
// transposed (16 keys of one query per lane), maximum and sum in-lane plus one half-wave
// exchange, W^T += V^T P^T with P used in place.  Dense layout, single pass (no key chunks).
#include "elsa_common.hpp"

namespace elsa {

__device__ __forceinline__ f32x16 mfma32s(float a, float b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

// MB consecutive elements of type T at byte offset voff + soff of a buffer, widened to float
template <typename T, int MB> struct Frag;
template <> struct Frag<float, 1> {
    static __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t r, int voff, int soff, float *o) {
        o[0] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, 0));
    }
};
template <> struct Frag<float, 2> {
    static __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t r, int voff, int soff, float *o) {
        const f32x2 x = __builtin_bit_cast(f32x2, __builtin_amdgcn_raw_buffer_load_b64(r, voff, soff, 0));
        o[0] = x[0]; o[1] = x[1];
    }
};
template <> struct Frag<float, 4> {
    static __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t r, int voff, int soff, float *o) {
        const f32x4 x = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, 0));
        o[0] = x[0]; o[1] = x[1]; o[2] = x[2]; o[3] = x[3];
    }
};
template <> struct Frag<_Float16, 1> {
    static __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t r, int voff, int soff, float *o) {
        o[0] = (float)__builtin_bit_cast(_Float16, __builtin_amdgcn_raw_buffer_load_b16(r, voff, soff, 0));
    }
};
template <> struct Frag<_Float16, 2> {
    static __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t r, int voff, int soff, float *o) {
        typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
        const f16x2 x = __builtin_bit_cast(f16x2, __builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, 0));
        o[0] = (float)x[0]; o[1] = (float)x[1];
    }
};
template <> struct Frag<_Float16, 4> {
    static __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t r, int voff, int soff, float *o) {
        const f16x4 x = __builtin_bit_cast(f16x4, __builtin_amdgcn_raw_buffer_load_b64(r, voff, soff, 0));
        o[0] = (float)x[0]; o[1] = (float)x[1]; o[2] = (float)x[2]; o[3] = (float)x[3];
    }
};

template <int D, typename T, int NQ>
__global__ __launch_bounds__(256, (D == 128 ? 1 : (D == 32 && NQ == 1) ? 4 : 2)) void fwd_mfma_small_kernel(FwdParams p) {
    constexpr int MB = D / 32;
    constexpr int ES = (int)sizeof(T);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int j = lane & 31, h = lane >> 5;

    // four independent work items per block: consecutive query tiles of a head sit side by side
    const long long total = (long long)p.q_tiles * p.B * p.H;
    const long long w = (long long)blockIdx.x * 4 + wave;
    if (w >= total) return;                      // no barrier anywhere in this kernel
    const int qt = (int)(w % p.q_tiles);
    const long long bh = w / p.q_tiles;
    const int n = p.n;
    int L = n;
    if (p.kv_len) L = min(max(p.kv_len[bh / p.H], 0), n);
    const int q0 = qt * 32 * NQ;
    const int kend = p.causal ? min(L, q0 + 32 * NQ) : L;
    const long long head_off = bh * (long long)n * D;

    float qf[NQ][D / 2];
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        const int row = q0 + nq * 32 + j;
#pragma unroll
        for (int cc = 0; cc < D / 8; ++cc) {
            f32x4 x = {0.f, 0.f, 0.f, 0.f};
            if (row < n) x = Io<T>::load4(p.q, head_off + (long long)row * D + 8 * cc + 4 * h);
#pragma unroll
            for (int t = 0; t < 4; ++t) qf[nq][4 * cc + t] = x[t] * p.qscale;
        }
    }

    float mrun[NQ], srun[NQ];
    f32x16 oacc[NQ][MB];
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        mrun[nq] = -INFINITY;
        srun[nq] = 0.f;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int i = 0; i < 16; ++i) oacc[nq][mb][i] = 0.f;
    }

    // rows at or beyond kend read as zero (and are masked)
    const long long slice_bytes = (long long)kend * D * ES;
    const __amdgpu_buffer_rsrc_t krs = make_rsrc(static_cast<const T *>(p.k) + head_off, slice_bytes);
    const __amdgpu_buffer_rsrc_t vrs = make_rsrc(static_cast<const T *>(p.v) + head_off, slice_bytes);
    const int kvoff = (j * D + 4 * h) * ES;          // K fragment: row j of the step, columns 8cc + 4h ..
    const int vvoff = (4 * h * D + MB * j) * ES;     // V fragment: key 8g + 4h + t, columns MB*j ..

    const int nsteps = (kend + 31) / 32;
    for (int st = 0; st < nsteps; ++st) {
        const int kg = st * 32;
        const int soff = kg * D * ES;

        float kfr[D / 8][4];
#pragma unroll
        for (int cc = 0; cc < D / 8; ++cc) Frag<T, 4>::load(krs, kvoff + 8 * cc * ES, soff, kfr[cc]);
        float vfr[16][MB];
#pragma unroll
        for (int i = 0; i < 16; ++i) Frag<T, MB>::load(vrs, vvoff + (8 * (i >> 2) + (i & 3)) * D * ES, soff, vfr[i]);

        // S^T = K Q^T on two accumulation chains
        f32x16 sacc[NQ];
        {
            f32x16 part[NQ][2];
#pragma unroll
            for (int nq = 0; nq < NQ; ++nq)
#pragma unroll
                for (int a = 0; a < 2; ++a)
#pragma unroll
                    for (int i = 0; i < 16; ++i) part[nq][a][i] = 0.f;
#pragma unroll
            for (int cc = 0; cc < D / 8; ++cc)
#pragma unroll
                for (int tt = 0; tt < 4; ++tt)
#pragma unroll
                    for (int nq = 0; nq < NQ; ++nq)
                        part[nq][cc / (D / 16)] = mfma32s(kfr[cc][tt], qf[nq][4 * cc + tt], part[nq][cc / (D / 16)]);
#pragma unroll
            for (int nq = 0; nq < NQ; ++nq) sacc[nq] = part[nq][0] + part[nq][1];
        }

        const bool need_mask = (kg + 32 > kend) || (p.causal && kg + 31 > q0);
        if (need_mask) {
#pragma unroll
            for (int nq = 0; nq < NQ; ++nq) {
                const int row = q0 + nq * 32 + j;
                const int lim = p.causal ? min(kend, row + 1) : kend;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int key = kg + 8 * (i >> 2) + 4 * h + (i & 3);
                    if (key >= lim) sacc[nq][i] = -INFINITY;
                }
            }
        }

#pragma unroll
        for (int nq = 0; nq < NQ; ++nq) {
            float mt = sacc[nq][0];
#pragma unroll
            for (int i = 1; i < 16; ++i) mt = fmaxf(mt, sacc[nq][i]);
            mt = half_max(mt);
            const float mnew = fmaxf(mrun[nq], mt);
            const float msafe = (mnew == -INFINITY) ? 0.f : mnew;
            if (__builtin_amdgcn_ballot_w64(mnew > mrun[nq]) != 0) {
                const float alpha = exp2_fast(mrun[nq] - msafe);
                srun[nq] *= alpha;
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) oacc[nq][mb][i] *= alpha;
                mrun[nq] = mnew;
            }
            float ps = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float e = exp2_fast(sacc[nq][i] - msafe);
                sacc[nq][i] = e;
                ps += e;
            }
            srun[nq] += ps;
        }

#pragma unroll
        for (int i = 0; i < 16; ++i)
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int nq = 0; nq < NQ; ++nq) oacc[nq][mb] = mfma32s(vfr[i][mb], sacc[nq][i], oacc[nq][mb]);
    }

#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        const int row = q0 + nq * 32 + j;
        const float stot = half_sum(srun[nq]);
        if (row >= n) continue;
        const float f = stot > 0.f ? 1.f / stot : 0.f;
        const long long obase = head_off + (long long)row * D;
        if (p.lse && h == 0) p.lse[bh * (long long)n + row] = lse_of(mrun[nq], stot);
        // register 4g+t of block mb is value column MB*(8g + 4h + t) + mb
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            float x[4 * MB];
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) x[t * MB + mb] = oacc[nq][mb][4 * g + t] * f;
#pragma unroll
            for (int c4 = 0; c4 < MB; ++c4)
                Io<T>::store4(p.out, obase + MB * (8 * g + 4 * h) + 4 * c4,
                              f32x4{x[4 * c4], x[4 * c4 + 1], x[4 * c4 + 2], x[4 * c4 + 3]});
        }
    }
}

template <int D, typename T, int NQ>
static int launch_small_one(const FwdParams &p, hipStream_t s) {
    const long long total = (long long)p.q_tiles * p.B * p.H;
    const long long blocks = (total + 3) / 4;
    if (blocks <= 0 || blocks > 0x7fffffffLL) return (int)hipErrorInvalidConfiguration;
    hipLaunchKernelGGL((fwd_mfma_small_kernel<D, T, NQ>), dim3((unsigned)blocks), dim3(256), 0, s, p);
    return (int)hipGetLastError();
}

template <int D, typename T>
static int launch_small_d(const FwdParams &p, int nq, hipStream_t s) {
    return nq == 2 ? launch_small_one<D, T, 2>(p, s) : launch_small_one<D, T, 1>(p, s);
}

// nq = 1: 32 query rows per wave, nq = 2: 64.  Dense layout, num_splits == 1, no partial states.
int launch_fwd_mfma_small(const FwdParams &p, int d, int f16, int nq, hipStream_t s) {
    if (p.cu_seqlens || p.num_splits != 1 || p.emit_partials) return (int)hipErrorInvalidValue;
    if (d == 32) return f16 ? launch_small_d<32, _Float16>(p, nq, s) : launch_small_d<32, float>(p, nq, s);
    if (d == 64) return f16 ? launch_small_d<64, _Float16>(p, nq, s) : launch_small_d<64, float>(p, nq, s);
    if (d == 128) return f16 ? launch_small_d<128, _Float16>(p, nq, s) : launch_small_d<128, float>(p, nq, s);
    return (int)hipErrorInvalidValue;
}

}  // namespace elsa
