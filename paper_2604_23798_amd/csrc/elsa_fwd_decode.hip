// ELSA forward for a handful of queries against a long key range (decoding against a cache,
// speculative steps): FP32 vector arithmetic, bound by the HBM reads of K and V.
//
// With one to four queries a 32-column matrix-core tile would spend 1/32 .. 1/8 of its work on
// real rows, so this kernel forms the scores on the vector ALU instead.  A key row of d elements
// is spread over LPR lanes (d/8 lanes of 8 columns each for d = 32, 64, 128; 4 lanes of 24 columns
// for d = 96; 16 lanes of 16 columns for d = 256; a lane's columns come in 16-byte pieces that lie
// 16*LPR bytes apart), so one wave instruction reads 16*LPR contiguous bytes of each of 64/LPR
// consecutive rows, fully coalesced; a lane multiplies its columns into the query, the LPR
// lanes of a key add their partial sums with DPP row operations (no LDS), and every lane folds
// the (key, score) pair into its OWN monoid state (m, S, W[8 columns]) with the merge operator of
// Eq. 3.  Lanes, waves and -- through the chunk states of Prop. 1 -- blocks cover disjoint key
// subsets.  At the end the lane states of a wave merge in registers, a log-depth tree of the same
// operator over DPP rotations, one crossbar swizzle and the half-wave swap; the four wave states
// meet in LDS, those of different blocks in the combine kernel.
#include <type_traits>

#include "elsa_common.hpp"

namespace elsa {

namespace {

template <int CTRL> __device__ __forceinline__ float dpp_get(float x) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xF, 0xF, true));
}
// sum over the LPR (4, 8 or 16) consecutive lanes of a key; every lane of the group gets the sum
template <int LPR> __device__ __forceinline__ float group_sum(float x) {
    x += dpp_get<0xB1>(x);                          // quad_perm [1,0,3,2]
    x += dpp_get<0x4E>(x);                          // quad_perm [2,3,0,1]: quads are uniform now
    if constexpr (LPR >= 8) x += dpp_get<0x141>(x);  // row_half_mirror: the other quad of each 8
    if constexpr (LPR >= 16) x += dpp_get<0x140>(x); // row_mirror: the other 8 of each 16
    return x;
}

// Value of the lane `STRIDE` away: a rotation inside the 16-lane row for 4 and 8 (DPP), the lane
// l ^ 16 (LDS crossbar swizzle, no memory) and the lane l ^ 32 (half-wave swap).
template <int STRIDE> __device__ __forceinline__ float lane_far(float x, int lane) {
    if constexpr (STRIDE == 4) return dpp_get<0x124>(x);         // row_ror:4
    else if constexpr (STRIDE == 8) return dpp_get<0x128>(x);    // row_ror:8
    else if constexpr (STRIDE == 16)
        return __builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, x), 0x401F));
    else {
        const unsigned u = __float_as_uint(x);
        auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
        return __uint_as_float(lane < 32 ? r[1] : r[0]);
    }
}

// Base and range are the same in every lane; saying so (v_readfirstlane) keeps the descriptor in
// scalar registers -- without it the compiler treats it as lane-dependent here and wraps every load
// in a loop over the distinct descriptor values.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc_uniform(const void *base, long long bytes) {
    const unsigned long long b = reinterpret_cast<unsigned long long>(base);
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)b);
    const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(b >> 32));
    const int nrec = __builtin_amdgcn_readfirstlane(bytes > 0 ? (int)(bytes < 0x7fffffffLL ? bytes : 0x7fffffffLL) : 0);
    return __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void *>(((unsigned long long)hi << 32) | lo), 0, nrec, 0x00020000);
}

// One 16-byte piece of a row (4 floats or 8 halves), widened to float.  AUX = 2 marks the load
// non-temporal (nt): K and V are read exactly once, and the hint keeps the stream from displacing
// cache lines on its way -- measured on 2.7 GB read by 1280 blocks: 6.13 TB/s plain, 6.95 TB/s nt.
template <typename T, int AUX> struct Piece;
template <int AUX> struct Piece<float, AUX> {
    static constexpr int W = 4;
    static __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t r, int voff, int soff, float *o) {
        const f32x4 a = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, AUX));
#pragma unroll
        for (int t = 0; t < 4; ++t) o[t] = a[t];
    }
};
template <int AUX> struct Piece<_Float16, AUX> {
    static constexpr int W = 8;
    static __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t r, int voff, int soff, float *o) {
        const f16x8 a = __builtin_bit_cast(f16x8, __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, AUX));
#pragma unroll
        for (int t = 0; t < 8; ++t) o[t] = (float)a[t];
    }
};

}  // namespace

template <int D, typename T, int NQ>
__global__ __launch_bounds__(256, (NQ == 1 && D != 96 && D != 256) ? 5 : NQ == 8 ? 2 : 1) void fwd_decode_kernel(FwdParams p) {
    constexpr int LPR = D == 96 ? 4 : D == 256 ? 16 : D / 8;   // lanes per key row (a power of two <= 16)
    constexpr int CPL = D / LPR;         // columns per lane: 8, 16 or 24
    constexpr int KPI = 64 / LPR;        // keys per wave instruction
    constexpr int U = CPL == 8 ? 4 : 2;  // key groups in flight per wave
    constexpr int ES = (int)sizeof(T);
    constexpr int NS = 2 + CPL;          // floats of state per (lane, query): m, S, W[CPL]
    // A lane owns CPL/PW pieces of PW columns (16 bytes) of its key row, piece c at columns
    // c*PW*LPR + PW*cs: the LPR lanes of a row then read 16*LPR contiguous bytes per instruction
    // (whole rows when a lane has one piece), i.e. whole 128-byte lines -- which is what lets the
    // loads be non-temporal: a line that two instructions share would be fetched twice.
    constexpr int PW = 16 / ES;
    constexpr int NP = CPL / PW;
    constexpr bool FULL_LINES = NP == 1 || LPR * 16 >= 128;
    using Pc = Piece<T, FULL_LINES ? 2 : 0>;
    static_assert(CPL % 8 == 0 && LPR * CPL == D && (CPL == 8 || NQ == 1), "unsupported shape");
    auto col = [](int lane_cs, int t) { return (t / PW) * PW * LPR + PW * lane_cs + t % PW; };
    __shared__ float st[4 * LPR * NQ * NS];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int cs = lane % LPR, ksub = lane / LPR;

    const Work wi = decode_work<D>(p);   // dense layout only (checked by the launcher)
    if (!wi.valid) return;               // uniform over the block
    const int c = wi.c;
    const long long bh = wi.bh;
    const int n = wi.n;
    const int coff = wi.coff;
    int L = wi.nk;
    if (p.kv_len) L = min(max(p.kv_len[bh / p.H], 0), wi.nk);
    const int q0 = wi.qt * NQ;
    // every lane of the block works on the same key range: scalar registers for the bounds
    const int kbeg = __builtin_amdgcn_readfirstlane(c * p.chunk);
    int kend = min(kbeg + p.chunk, L);
    if (p.causal) kend = min(kend, q0 + NQ + coff);
    kend = __builtin_amdgcn_readfirstlane(kend);

    float qr[NQ][CPL];
    int lim[NQ];                         // first key the query cannot see
#pragma unroll
    for (int iq = 0; iq < NQ; ++iq) {
        const int row = q0 + iq;
#pragma unroll
        for (int c4 = 0; c4 < CPL / 4; ++c4) {
            f32x4 a = {0.f, 0.f, 0.f, 0.f};
            if (row < n) a = Io<T>::load4(p.q, wi.base + (long long)row * D + col(cs, 4 * c4));
#pragma unroll
            for (int t = 0; t < 4; ++t) qr[iq][4 * c4 + t] = a[t] * p.qscale;
        }
        lim[iq] = p.causal ? min(kend, row + 1 + coff) : kend;
    }
    int lim_min = lim[0];
#pragma unroll
    for (int iq = 1; iq < NQ; ++iq) lim_min = min(lim_min, lim[iq]);

    float m[NQ], S[NQ], W[NQ][CPL];
#pragma unroll
    for (int iq = 0; iq < NQ; ++iq) {
        m[iq] = -INFINITY;
        S[iq] = 0.f;
#pragma unroll
        for (int t = 0; t < CPL; ++t) W[iq][t] = 0.f;
    }

    // rows at or beyond kend read as zero and are masked
    const long long slice_bytes = kend > 0 ? (long long)kend * D * ES : 0;
    const __amdgpu_buffer_rsrc_t krs = make_rsrc_uniform(static_cast<const T *>(p.k) + wi.kbase, slice_bytes);
    const __amdgpu_buffer_rsrc_t vrs = make_rsrc_uniform(static_cast<const T *>(p.v) + wi.kbase, slice_bytes);
    const int voff = (ksub * D + PW * cs) * ES;          // piece 0; piece c is 16*LPR bytes further

    // the four waves take turns on runs of U key groups, so that the block reads one contiguous
    // stream of 4*U*KPI rows per round
    const int ngroups = kend > kbeg ? (kend - kbeg + KPI - 1) / KPI : 0;
    for (int g0 = wave * U; g0 < ngroups; g0 += 4 * U) {
        float kf[U][CPL], vf[U][CPL];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            // groups past the chunk start at or beyond kend: every lane reads zeros there
            const int key0 = min(kbeg + (g0 + u) * KPI, kend);
            const int soff = __builtin_amdgcn_readfirstlane(key0 * D * ES);
#pragma unroll
            for (int c = 0; c < NP; ++c) {
                Pc::load(krs, voff + c * 16 * LPR, soff, kf[u] + PW * c);
                Pc::load(vrs, voff + c * 16 * LPR, soff, vf[u] + PW * c);
            }
        }
        const bool need_mask = kbeg + (g0 + U) * KPI > lim_min;
#pragma unroll
        for (int iq = 0; iq < NQ; ++iq) {
            float s[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float acc = qr[iq][0] * kf[u][0];
#pragma unroll
                for (int t = 1; t < CPL; ++t) acc = fmaf(qr[iq][t], kf[u][t], acc);
                s[u] = group_sum<LPR>(acc);
            }
            if (need_mask) {
#pragma unroll
                for (int u = 0; u < U; ++u)
                    if (kbeg + (g0 + u) * KPI + ksub >= lim[iq]) s[u] = -INFINITY;
            }
            float mt = s[0];
#pragma unroll
            for (int u = 1; u < U; ++u) mt = fmaxf(mt, s[u]);
            const float mnew = fmaxf(m[iq], mt);
            const float msafe = (mnew == -INFINITY) ? 0.f : mnew;   // identity (+) identity = identity
            const float alpha = exp2_fast(m[iq] - msafe);
            m[iq] = mnew;
            float e[U], ps = 0.f;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                e[u] = exp2_fast(s[u] - msafe);
                ps += e[u];
            }
            S[iq] = S[iq] * alpha + ps;
#pragma unroll
            for (int t = 0; t < CPL; ++t) {
                float w = W[iq][t] * alpha;
#pragma unroll
                for (int u = 0; u < U; ++u) w = fmaf(e[u], vf[u][t], w);
                W[iq][t] = w;
            }
        }
    }

    // ---- in-register tree over the KPI lanes of the wave that share a column slice (log2 KPI levels
    // of Eq. 3: lanes 4, 8 away inside the row by DPP rotations, 16 and 32 away across the rows);
    // afterwards the lanes of key group 0 hold the wave's state
    auto tree_level = [&](auto stride_tag) __attribute__((always_inline)) {
        constexpr int STRIDE = decltype(stride_tag)::value;
#pragma unroll
        for (int iq = 0; iq < NQ; ++iq) {
            const float mo = lane_far<STRIDE>(m[iq], lane);
            const float So = lane_far<STRIDE>(S[iq], lane);
            float fa, fb;
            m[iq] = merge_factors(m[iq], mo, fa, fb);
            S[iq] = S[iq] * fa + So * fb;
#pragma unroll
            for (int t = 0; t < CPL; ++t) W[iq][t] = W[iq][t] * fa + lane_far<STRIDE>(W[iq][t], lane) * fb;
        }
    };
    if constexpr (LPR <= 4) tree_level(std::integral_constant<int, 4>{});
    if constexpr (LPR <= 8) tree_level(std::integral_constant<int, 8>{});
    tree_level(std::integral_constant<int, 16>{});
    tree_level(std::integral_constant<int, 32>{});

    // ---- the four wave states meet in LDS
    if (ksub == 0) {
#pragma unroll
        for (int iq = 0; iq < NQ; ++iq) {
            float *dst = &st[((wave * LPR + cs) * NQ + iq) * NS];
            dst[0] = m[iq];
            dst[1] = S[iq];
#pragma unroll
            for (int t = 0; t < CPL; ++t) dst[2 + t] = W[iq][t];
        }
    }
    __syncthreads();
    if (tid >= LPR * NQ) return;         // the LPR * NQ <= 128 threads below meet no further barrier
    const int iq = tid / LPR, cs2 = tid % LPR;
    const int row = q0 + iq;
    if (row >= n) return;
    float ma = -INFINITY, Sa = 0.f, Wa[CPL];
#pragma unroll
    for (int t = 0; t < CPL; ++t) Wa[t] = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const float *src = &st[((w * LPR + cs2) * NQ + iq) * NS];
        float fa, fb;
        ma = merge_factors(ma, src[0], fa, fb);
        Sa = Sa * fa + src[1] * fb;
#pragma unroll
        for (int t = 0; t < CPL; ++t) Wa[t] = Wa[t] * fa + src[2 + t] * fb;
    }
    if (p.emit_partials) {
        const long long prow = (bh * p.num_splits + c) * (long long)n + row;
        float fn = 1.f, fold = 0.f;
        if (p.accumulate) {                      // stored (+) new, Eq. 3; the LPR threads of a row all read first
            const float ms = p.part_m[prow], Ss = p.part_S[prow];
            ma = merge_factors(ma, ms, fn, fold);
            Sa = Sa * fn + Ss * fold;
        }
        if (cs2 == 0) {
            p.part_m[prow] = p.m_natural ? ma * kLn2 : ma;
            p.part_S[prow] = Sa;
        }
#pragma unroll
        for (int c4 = 0; c4 < CPL / 4; ++c4) {
            const long long at = prow * D + col(cs2, 4 * c4);
            f32x4 x = f32x4{Wa[4 * c4], Wa[4 * c4 + 1], Wa[4 * c4 + 2], Wa[4 * c4 + 3]} * fn;
            if (p.accumulate) x += Io<float>::load4(p.part_W, at) * fold;
            Io<float>::store4(p.part_W, at, x);
        }
    } else {
        const float f = Sa > 0.f ? 1.f / Sa : 0.f;
        if (p.lse && cs2 == 0) p.lse[bh * (long long)n + row] = lse_of(ma, Sa);
        const long long o = wi.base + (long long)row * D;
#pragma unroll
        for (int c4 = 0; c4 < CPL / 4; ++c4)
            Io<T>::store4(p.out, o + col(cs2, 4 * c4), f32x4{Wa[4 * c4] * f, Wa[4 * c4 + 1] * f, Wa[4 * c4 + 2] * f, Wa[4 * c4 + 3] * f});
    }
}

template <int D, typename T, int NQ>
static int launch_decode_one(const FwdParams &p, hipStream_t s) {
    const long long total = (long long)p.q_tiles * p.B * p.H * p.num_splits;
    long long blocks = total;
    if (p.xcd_map == 2) blocks = (total + kNumXcd - 1) / kNumXcd * kNumXcd;
    if (blocks <= 0 || blocks > 0x7fffffffLL) return (int)hipErrorInvalidConfiguration;
    hipLaunchKernelGGL((fwd_decode_kernel<D, T, NQ>), dim3((unsigned)blocks), dim3(256), 0, s, p);
    return (int)hipGetLastError();
}

template <int D, typename T>
static int launch_decode_d(const FwdParams &p, int nq, hipStream_t s) {
    if constexpr (D == 96 || D == 256) {         // wide lanes: one query per block only
        return nq == 1 ? launch_decode_one<D, T, 1>(p, s) : (int)hipErrorInvalidValue;
    } else {
        if constexpr (D == 128 && std::is_same<T, float>::value) {
            if (nq == 8) return launch_decode_one<D, T, 8>(p, s);
        }
        if (nq == 8) return (int)hipErrorInvalidValue;
        return nq == 1 ? launch_decode_one<D, T, 1>(p, s) : launch_decode_one<D, T, 4>(p, s);
    }
}

// nq = 1, 4 or 8 (FP32, d = 128) queries per block (p.tq must say the same).  Dense layout only.
int launch_fwd_decode(const FwdParams &p, int d, int f16, int nq, hipStream_t s) {
    if (p.cu_seqlens || (nq != 1 && nq != 4 && nq != 8) || p.tq != nq) return (int)hipErrorInvalidValue;
    if (d == 32) return f16 ? launch_decode_d<32, _Float16>(p, nq, s) : launch_decode_d<32, float>(p, nq, s);
    if (d == 64) return f16 ? launch_decode_d<64, _Float16>(p, nq, s) : launch_decode_d<64, float>(p, nq, s);
    if (d == 128) return f16 ? launch_decode_d<128, _Float16>(p, nq, s) : launch_decode_d<128, float>(p, nq, s);
    if (d == 96) return f16 ? launch_decode_d<96, _Float16>(p, nq, s) : launch_decode_d<96, float>(p, nq, s);
    if (d == 256) return f16 ? launch_decode_d<256, _Float16>(p, nq, s) : launch_decode_d<256, float>(p, nq, s);
    return (int)hipErrorInvalidValue;
}

}  // namespace elsa
