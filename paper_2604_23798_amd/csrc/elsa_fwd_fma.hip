// ELSA forward, FP32 vector-FMA path (gfx950).  Kept beside the MFMA path so that the two
// can be measured against each other; it never touches the matrix cores.
//
// Every lane owns one query row and runs the per-query fold of Alg. 1 over the keys of
// its wave: the K and V rows are wave-uniform, so they are fetched through uniform
// (scalar) loads and enter the FMAs as scalar operands -- no LDS traffic, no cross-lane
// step.  Keys are taken G at a time so the running state is rescaled once per group
// (the merge operator applied to the group's state) instead of once per key.  The WK
// waves of a block that split the key range merge their states through LDS.
#include <type_traits>

#include "elsa_common.hpp"

namespace elsa {

template <typename T> __device__ __forceinline__ float ld_uniform(const T *p, int t) { return (float)p[t]; }

template <int D, typename T, int WQ, int WK, int WPE>
__global__ __launch_bounds__(64 * WQ * WK, WPE) void fwd_fma_kernel(FwdParams p) {
    constexpr int TQ = 64 * WQ;
    constexpr int G = 4;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wq = wave % WQ, wk = wave / WQ;

    const Work wi = decode_work<D>(p);
    if (!wi.valid) return;
    const int qt = wi.qt, c = wi.c;
    const long long bh = wi.bh;
    const int n = wi.n;
    const long long ts = wi.ts;          // elements between consecutive tokens
    const int coff = wi.coff;            // causal: key j visible to row i iff j <= i + coff
    int L = wi.nk;
    if (p.kv_len) L = min(max(p.kv_len[bh / p.H], 0), wi.nk);
    const int q0 = qt * TQ;
    const int kbeg = c * p.chunk;
    int kend = min(kbeg + p.chunk, L);
    if (p.causal) kend = min(kend, q0 + TQ + coff);

    // this wave's slice of the block's key range
    const int span = kend > kbeg ? kend - kbeg : 0;
    const int per = (span + WK - 1) / WK;
    const int wbeg = kbeg + wk * per;
    int wend = min(wbeg + per, kend);
    const int wrow0 = q0 + wq * 64;
    if (p.causal) wend = min(wend, wrow0 + 64 + coff);

    const long long head_off = wi.base;
    const int row = wrow0 + lane;
    const int lim = p.causal ? min(wend, row + 1 + coff) : wend;      // keys >= lim are invisible to this row

    float qr[D];
#pragma unroll
    for (int c4 = 0; c4 < D / 4; ++c4) {
        f32x4 x = {0.f, 0.f, 0.f, 0.f};
        if (row < n) x = Io<T>::load4(p.q, head_off + (long long)row * ts + 4 * c4);
#pragma unroll
        for (int t = 0; t < 4; ++t) qr[4 * c4 + t] = x[t] * p.qscale;
    }

    float m = -INFINITY, S = 0.f;
    float W[D];
#pragma unroll
    for (int t = 0; t < D; ++t) W[t] = 0.f;

    const T *__restrict__ kp = static_cast<const T *>(p.k) + wi.kbase;
    const T *__restrict__ vp = static_cast<const T *>(p.v) + wi.kbase;

    // One group of G keys merged into the state (Eq. 3 with the group's state).  TAIL: the group sticks out of the
    // wave's range -- keys at or beyond wend are the identity for every row and are skipped, not multiplied by a
    // zero weight (their rows may be padding that holds anything, NaN and Inf included).
    auto group = [&](int j0, auto tail_tag) __attribute__((always_inline)) {
        constexpr bool TAIL = decltype(tail_tag)::value;
        float s[G];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            s[g] = -INFINITY;
            if (TAIL && j0 + g >= wend) continue;
            const T *__restrict__ kj = kp + (long long)(j0 + g) * ts;
            float acc = 0.f;
#pragma unroll
            for (int t = 0; t < D; ++t) acc = fmaf(qr[t], ld_uniform(kj, t), acc);
            if (j0 + g < lim) s[g] = acc;
        }
        float mt = s[0];
#pragma unroll
        for (int g = 1; g < G; ++g) mt = fmaxf(mt, s[g]);
        const float mnew = fmaxf(m, mt);
        const float msafe = (mnew == -INFINITY) ? 0.f : mnew;
        const float alpha = exp2_fast(m - msafe);
        m = mnew;
        float e[G], ps = 0.f;
#pragma unroll
        for (int g = 0; g < G; ++g) {
            e[g] = exp2_fast(s[g] - msafe);
            ps += e[g];
        }
        S = S * alpha + ps;
#pragma unroll
        for (int t = 0; t < D; ++t) W[t] *= alpha;
#pragma unroll
        for (int g = 0; g < G; ++g) {
            if (TAIL && j0 + g >= wend) continue;
            const T *__restrict__ vj = vp + (long long)(j0 + g) * ts;
#pragma unroll
            for (int t = 0; t < D; ++t) W[t] = fmaf(e[g], ld_uniform(vj, t), W[t]);
        }
    };
    int j0 = wbeg;
    for (; j0 + G <= wend; j0 += G) group(j0, std::false_type{});
    if (j0 < wend) group(j0, std::true_type{});

    if constexpr (WK > 1) {
        extern __shared__ __align__(16) float smem[];
        constexpr int NS = D + 2;
#pragma unroll
        for (int s = WK / 2; s >= 1; s >>= 1) {
            if (wk >= s && wk < 2 * s) {
                float *dst = smem + ((wk - s) * WQ + wq) * NS * 64 + lane;
                dst[0] = m;
                dst[64] = S;
#pragma unroll
                for (int t = 0; t < D; ++t) dst[64 * (2 + t)] = W[t];
            }
            __syncthreads();
            if (wk < s) {
                const float *src = smem + (wk * WQ + wq) * NS * 64 + lane;
                const float mb = src[0], sb = src[64];
                const float mnew = fmaxf(m, mb);
                const float msafe = (mnew == -INFINITY) ? 0.f : mnew;
                const float fa = exp2_fast(m - msafe), fb = exp2_fast(mb - msafe);
                m = mnew;
                S = S * fa + sb * fb;
#pragma unroll
                for (int t = 0; t < D; ++t) W[t] = W[t] * fa + src[64 * (2 + t)] * fb;
            }
            __syncthreads();
        }
        if (wk != 0) return;
    }

    if (row >= n) return;
    if (p.emit_partials) {
        const long long prow = (bh * p.num_splits + c) * (long long)n + row;
        float fn = 1.f, fold = 0.f;
        if (p.accumulate) {                      // stored (+) new, Eq. 3
            const float ms = p.part_m[prow], Ss = p.part_S[prow];
            m = merge_factors(m, ms, fn, fold);
            S = S * fn + Ss * fold;
        }
        p.part_m[prow] = p.m_natural ? m * kLn2 : m;
        p.part_S[prow] = S;
#pragma unroll
        for (int c4 = 0; c4 < D / 4; ++c4) {
            f32x4 x = f32x4{W[4 * c4], W[4 * c4 + 1], W[4 * c4 + 2], W[4 * c4 + 3]} * fn;
            if (p.accumulate) x += Io<float>::load4(p.part_W, prow * D + 4 * c4) * fold;
            Io<float>::store4(p.part_W, prow * D + 4 * c4, x);
        }
    } else {
        const float f = S > 0.f ? 1.f / S : 0.f;
        if (p.lse) p.lse[bh * (long long)n + row] = lse_of(m, S);
#pragma unroll
        for (int c4 = 0; c4 < D / 4; ++c4)
            Io<T>::store4(p.out, head_off + (long long)row * ts + 4 * c4,
                          f32x4{W[4 * c4] * f, W[4 * c4 + 1] * f, W[4 * c4 + 2] * f, W[4 * c4 + 3] * f});
    }
}

// 3, 4, 5: one / four / eight queries per block against a long key range (elsa_fwd_decode.hip; eight: FP32, d = 128)
static const char *kFmaNames[kFmaVariants] = {"fma_q256_w4", "fma_q64_xw4", "fma_decode_q1", "fma_decode_q4", "fma_decode_q8"};
int fma_variant_tq(int variant, int) {
    return variant == 1 ? 256 : variant == 2 ? 64 : variant == 3 ? 1 : variant == 4 ? 4 : variant == 5 ? 8 : 0;
}
const char *fma_variant_name(int variant) {
    return (variant >= 1 && variant <= kFmaVariants) ? kFmaNames[variant - 1] : nullptr;
}

template <int D, typename T, int WQ, int WK, int WPE>
static int launch_one(const FwdParams &p, hipStream_t s) {
    constexpr size_t smem = WK > 1 ? (size_t)(WK / 2) * WQ * (D + 2) * 64 * sizeof(float) : 0;
    auto kern = fwd_fma_kernel<D, T, WQ, WK, WPE>;
    static bool attr_done[kMaxDevices] = {};   // per instantiation and device
    if (smem > 0) {
        if (hipError_t e = allow_dynamic_lds(kern, smem, attr_done); e != hipSuccess) return (int)e;
    }
    const long long total = p.cu_seqlens ? (long long)p.var_tiles * p.H : (long long)p.q_tiles * p.B * p.H * p.num_splits;
    long long blocks = total;
    if (p.xcd_map == 2 && !p.cu_seqlens) blocks = (total + kNumXcd - 1) / kNumXcd * kNumXcd;
    if (blocks <= 0 || blocks > 0x7fffffffLL) return (int)hipErrorInvalidConfiguration;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(64 * WQ * WK), smem, s, p);
    return (int)hipGetLastError();
}

template <int D, typename T>
static int launch_variant(const FwdParams &p, int variant, hipStream_t s) {
    switch (variant) {
        // d = 128 keeps 256 state registers per lane: one wave per SIMD
        case 1: return launch_one<D, T, 4, 1, (D <= 64 ? 2 : 1)>(p, s);
        case 2: return launch_one<D, T, 1, 4, (D <= 64 ? 2 : 1)>(p, s);
        default: return (int)hipErrorInvalidValue;
    }
}

int launch_fwd_fma(const FwdParams &p, int d, int f16, int variant, hipStream_t s, const char **name) {
    if (name) *name = fma_variant_name(variant);
    if (variant >= 3 && variant <= 5) return launch_fwd_decode(p, d, f16, variant == 3 ? 1 : variant == 4 ? 4 : 8, s);
    if (d == 32) return f16 ? launch_variant<32, _Float16>(p, variant, s) : launch_variant<32, float>(p, variant, s);
    if (d == 64) return f16 ? launch_variant<64, _Float16>(p, variant, s) : launch_variant<64, float>(p, variant, s);
    if (d == 128) return f16 ? launch_variant<128, _Float16>(p, variant, s) : launch_variant<128, float>(p, variant, s);
    return (int)hipErrorInvalidValue;
}

}  // namespace elsa
