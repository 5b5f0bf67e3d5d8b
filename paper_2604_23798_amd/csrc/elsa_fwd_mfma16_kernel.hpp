// ELSA forward, FP16-I/O path on the FP16 matrix cores (gfx950), FP32 state.
//
// Same tiling and the same monoid fold as the FP32 MFMA kernel, with
// v_mfma_f32_32x32x16_f16 for both contractions: Q, K, V stay FP16 (exact inputs), every
// score, the running maximum m, the normaliser S and the weighted sum W are FP32, and the
// exponentials are rounded to FP16 (nearest-even) only as the B operand of the PV product.
// 16-bit MFMA operands are contiguous along the contraction index.  K (contraction over d) is
// staged row-major and read with 16-byte LDS reads.  V (contraction over keys) is staged row-major
// too and its fragments are fetched with the transposing LDS read ds_read_b64_tr_b16: in every
// group of 16 lanes, lane 4e+a supplies the address of four consecutive value columns of key e,
// and lane i receives column i of keys 0..3 -- exactly the V^T fragment of 16 value columns x 4
// keys.  The contraction index of PV is permuted so that the 8 exponentials a lane already holds
// in accumulator registers 8u..8u+7 are its B operand as they are.
// Scores stay in raw units (q.k); scale*log2(e) enters in the exponent, 2^(s*c - m*c), through
// one FMA per score, so no rounding of Q is added.  Requires scale != 0 (the caller falls back
// to the FP32-MFMA kernel otherwise).
#pragma once
#include "elsa_common.hpp"

namespace elsa {

typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ f32x16 mfma16(f16x8 a, f16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
}

// D: columns of q and k (the contraction of the scores); DV: columns of v and out (rows of W^T).
// TRIM: 0 = the fold as first written (comparison), 1 = fewer instructions per step (the steps of a tile are separate
// copies of the body, so LDS offsets are constants; one minimum instead of compare + select for rows that have seen no
// key; row sum started from the first weight), 2 = as 1, and the K fragments of the next step are requested early,
// 3 = as 2 with a lagging reference (below), 4 = as 1 with a lagging reference.
// Lagging reference (launches that write the output, not a state): the m of the running state is allowed to lag the
// true maximum.  (m, S, W) and (m', S e^(m-m'), W e^(m-m')) are the same element of the monoid and give the same W / S,
// so a step first forms its weights against the stored m and keeps them if every lane's partial row sum stays below
// kLagLimit (then no weight exceeds it either: no FP16 overflow, and a reference BELOW the true maximum only moves
// the weights away from the FP16 subnormals).  Otherwise -- the first keys of a row, a score more than ~2^10 above the
// stored reference, a NaN -- the step is redone the exact way: maximum, rescale, new reference.  This removes the
// row maximum (10 instructions), its half-wave exchange and test (4) from nearly every step.
template <int D, int NQ, int WQ, int WK, int KS, int WPE, int DV = D, int TRIM = 4>
__global__ __launch_bounds__(64 * WQ * WK, WPE) void fwd_mfma16_kernel(FwdParams p) {
    constexpr int NT = 64 * WQ * WK;
    constexpr int TQ = 32 * NQ * WQ;
    constexpr int TKB = KS * WK;             // keys per LDS tile
    constexpr int KROWB = D * 2 + 16;        // bytes per K row: 16-byte reads of 32 rows hit distinct banks
    constexpr int VROWB = DV * 2 + 32;       // bytes per V row: the 4 rows x 32 bytes of a transposing read hit distinct banks
    constexpr int KBUFB = TKB * KROWB;
    constexpr int VBUFB = TKB * VROWB;
    constexpr int CPR = D / 8;               // 16-byte chunks per K row in HBM
    constexpr int CPRV = DV / 8;             // ... per V row
    constexpr int LPT = TKB * CPR / NT;      // staged chunks per thread, K
    constexpr int LPTV = TKB * CPRV / NT;    // ... V
    constexpr int MB = DV / 32;              // 32-row blocks of W^T
    constexpr int KC = D / 16;               // MFMAs per score tile
    static_assert(TKB * CPR % NT == 0 && TKB * CPRV % NT == 0, "tile must divide evenly over the threads");
    static_assert(D % 16 == 0 && DV % 32 == 0, "head dimensions");
    static_assert(KS % 32 == 0, "a wave consumes keys 32 at a time");

    extern __shared__ __align__(16) unsigned char smem_b[];
    unsigned char *Ks = smem_b;                      // [2][KBUFB]
    unsigned char *Vs = smem_b + 2 * KBUFB;          // [2][VBUFB]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wq = wave % WQ, wk = wave / WQ;
    const int j = lane & 31, h = lane >> 5;

    const Work wi = decode_work<D>(p);
    if (!wi.valid) return;
    const int qt = wi.qt, c = wi.c;
    const long long bh = wi.bh;
    const int n = wi.n;
    const long long ts = wi.ts;          // elements between consecutive tokens of Q and K
    const long long tsv = DV == D ? ts : ts / D * DV;   // ... of V and out
    const int coff = wi.coff;            // causal: key j visible to row i iff j <= i + coff
    int L = wi.nk;
    if (p.kv_len) L = min(max(p.kv_len[bh / p.H], 0), wi.nk);
    const int q0 = qt * TQ;
    const int kbeg = c * p.chunk;
    int kend = min(kbeg + p.chunk, L);
    if (p.causal) kend = min(kend, q0 + TQ + coff);
    const int ntiles = kend > kbeg ? (kend - kbeg + TKB - 1) / TKB : 0;

    const long long head_off = wi.base;   // Q
    const long long kv_off = wi.kbase;     // K
    const long long out_off = DV == D ? head_off : head_off / D * DV;
    const long long v_off = DV == D ? kv_off : kv_off / D * DV;
    const int wrow0 = q0 + wq * NQ * 32;
    const _Float16 *qp = static_cast<const _Float16 *>(p.q);
    const _Float16 *kp = static_cast<const _Float16 *>(p.k);
    const _Float16 *vp = static_cast<const _Float16 *>(p.v);

    // log2-unit score = (q.k) * qscale.  A negative scale is moved into Q (exact sign flip) so
    // that the maximum of the raw scores is the maximum of the scaled ones.
    const float cs = fabsf(p.qscale);
    const bool flip = p.qscale < 0.f;

    // ---- Q fragments (B operand): lane (j,h) holds columns 16*cc + 8*h .. +7 of query row j
    f16x8 qf[NQ][KC];
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        const int row = wrow0 + nq * 32 + j;
#pragma unroll
        for (int cc = 0; cc < KC; ++cc) {
            f16x8 x = {0, 0, 0, 0, 0, 0, 0, 0};
            if (row < n) x = *reinterpret_cast<const f16x8 *>(qp + head_off + (long long)row * ts + 16 * cc + 8 * h);
            if (flip) x = -x;
            qf[nq][cc] = x;
        }
    }

    constexpr bool LAG = TRIM >= 3;
    constexpr float kLagLimit = 1024.f;
    float mrun[NQ], srun[NQ];               // mrun in raw score units
    float nmcr[NQ];                         // LAG: -m*c of the stored reference (3e38 while the row has seen no key)
    f32x16 oacc[NQ][MB];
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        mrun[nq] = -INFINITY;
        srun[nq] = 0.f;
        nmcr[nq] = 3.0e38f;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int i = 0; i < 16; ++i) oacc[nq][mb][i] = 0.f;
    }

    // Tiles are fetched through buffer descriptors whose byte range ends with the last visible row
    // of the chunk: rows beyond it read as zero, the per-thread offsets are constants and the
    // tile's position is one scalar offset (no vector address arithmetic, no lane masks).
    f16x8 kst[LPT], vst[LPTV];
    const long long slice_bytes = kend > 0 ? ((long long)(kend - 1) * ts + D) * 2 : 0;
    const long long slice_bytes_v = kend > 0 ? ((long long)(kend - 1) * tsv + DV) * 2 : 0;
    const __amdgpu_buffer_rsrc_t krs = make_rsrc(kp + kv_off, slice_bytes);
    const __amdgpu_buffer_rsrc_t vrs = make_rsrc(vp + v_off, slice_bytes_v);
    int voff[LPT], voffv[LPTV];
#pragma unroll
    for (int i = 0; i < LPT; ++i) {
        const int e = tid + i * NT;
        voff[i] = (int)(((long long)(e / CPR) * ts + 8 * (e % CPR)) * 2);
    }
#pragma unroll
    for (int i = 0; i < LPTV; ++i) {
        const int e = tid + i * NT;
        voffv[i] = (int)(((long long)(e / CPRV) * tsv + 8 * (e % CPRV)) * 2);
    }
    auto gload = [&](int t) {
        const int soff = (int)((long long)(kbeg + t * TKB) * ts * 2);
        if constexpr (WK > 1) {
            // key-splitting tiles with a single query tile per head read K and V exactly once:
            // non-temporal loads (whole lines per instruction) keep the stream out of the caches' way
            if (p.kv_once) {
                const int soffv = (int)((long long)(kbeg + t * TKB) * tsv * 2);
#pragma unroll
                for (int i = 0; i < LPT; ++i)
                    kst[i] = __builtin_bit_cast(f16x8, __builtin_amdgcn_raw_buffer_load_b128(krs, voff[i], soff, 2));
#pragma unroll
                for (int i = 0; i < LPTV; ++i)
                    vst[i] = __builtin_bit_cast(f16x8, __builtin_amdgcn_raw_buffer_load_b128(vrs, voffv[i], soffv, 2));
                return;
            }
        }
        if constexpr (DV == D) {                // K and V loads interleaved
#pragma unroll
            for (int i = 0; i < LPT; ++i) {
                kst[i] = __builtin_bit_cast(f16x8, __builtin_amdgcn_raw_buffer_load_b128(krs, voff[i], soff, 0));
                vst[i] = __builtin_bit_cast(f16x8, __builtin_amdgcn_raw_buffer_load_b128(vrs, voff[i], soff, 0));
            }
        } else {
            const int soffv = (int)((long long)(kbeg + t * TKB) * tsv * 2);
#pragma unroll
            for (int i = 0; i < LPT; ++i)
                kst[i] = __builtin_bit_cast(f16x8, __builtin_amdgcn_raw_buffer_load_b128(krs, voff[i], soff, 0));
#pragma unroll
            for (int i = 0; i < LPTV; ++i)
                vst[i] = __builtin_bit_cast(f16x8, __builtin_amdgcn_raw_buffer_load_b128(vrs, voffv[i], soffv, 0));
        }
    };
    auto lstore = [&](int buf) {
#pragma unroll
        for (int i = 0; i < LPT; ++i) {
            const int e = tid + i * NT;
            const int row = e / CPR, c8 = e % CPR;
            *reinterpret_cast<f16x8 *>(Ks + buf * KBUFB + row * KROWB + 16 * c8) = kst[i];
            if constexpr (DV == D) *reinterpret_cast<f16x8 *>(Vs + buf * VBUFB + row * VROWB + 16 * c8) = vst[i];
        }
        if constexpr (DV != D) {
#pragma unroll
            for (int i = 0; i < LPTV; ++i) {
                const int e = tid + i * NT;
                const int row = e / CPRV, c8 = e % CPRV;
                *reinterpret_cast<f16x8 *>(Vs + buf * VBUFB + row * VROWB + 16 * c8) = vst[i];
            }
        }
    };

    if (ntiles > 0) {
        gload(0);
        lstore(0);
        __syncthreads();
    }
    const int wave_lim = p.causal ? min(kend, wrow0 + NQ * 32 + coff) : kend;
    for (int t = 0; t < ntiles; ++t) {
        const int buf = t & 1;
        if (t + 1 < ntiles) gload(t + 1);
        const unsigned char *Kb = Ks + buf * KBUFB;
        const unsigned char *Vb = Vs + buf * VBUFB;
        const int kg0 = kbeg + t * TKB + wk * KS;
        const int nact = min(KS / 32, max(0, (wave_lim - kg0 + 31) / 32));
        // TRIM: the steps of a tile are separate copies of the loop body, so that a step's place inside the tile is
        // a constant of its LDS reads (no address arithmetic per step)
        constexpr bool KPRE = TRIM == 2 || TRIM == 3;
        f16x8 kpre[KPRE ? KC : 1];
        auto step = [&](const int ks) __attribute__((always_inline)) {
            const int kl = wk * KS + ks * 32;
            const int kg = kg0 + ks * 32;

            // ---- (a1) S^T = K Q^T, raw units
            f32x16 sacc[NQ];
#pragma unroll
            for (int nq = 0; nq < NQ; ++nq)
#pragma unroll
                for (int i = 0; i < 16; ++i) sacc[nq][i] = 0.f;
            // the K fragments of the step are requested before the first MFMA that needs them: all of them,
            // or two at a time at d = 256 under the register cap of two waves per SIMD (sixteen fragments
            // there spilled 50 registers more and ran 2.9 times slower: 16.9 against 5.8 ms at H = 16,
            // n = 16384); the reads then overlap the MFMA chain instead of being waited for one by one
            constexpr int PF = (KC <= 12 || WPE == 1) ? KC : 2;
            // KPRE: the fragments of the NEXT step of the tile are requested as soon as this step's score MFMAs are
            // issued, so that their LDS latency passes under the fold instead of in front of the next MFMA chain
            // (the first step of a tile has to wait for the barrier and reads its own)
            if constexpr (KPRE) {
                if (ks == 0) {
#pragma unroll
                    for (int cc = 0; cc < KC; ++cc)
                        kpre[cc] = *reinterpret_cast<const f16x8 *>(Kb + (kl + j) * KROWB + 32 * cc + 16 * h);
                }
#pragma unroll
                for (int cc = 0; cc < KC; ++cc)
#pragma unroll
                    for (int nq = 0; nq < NQ; ++nq) sacc[nq] = mfma16(kpre[cc], qf[nq][cc], sacc[nq]);
                if (ks + 1 < KS / 32) {
#pragma unroll
                    for (int cc = 0; cc < KC; ++cc)
                        kpre[cc] = *reinterpret_cast<const f16x8 *>(Kb + (kl + 32 + j) * KROWB + 32 * cc + 16 * h);
                }
            } else {
#pragma unroll
            for (int c0 = 0; c0 < KC; c0 += PF) {
                f16x8 kf[PF];
#pragma unroll
                for (int cc = 0; cc < PF; ++cc)
                    kf[cc] = *reinterpret_cast<const f16x8 *>(Kb + (kl + j) * KROWB + 32 * (c0 + cc) + 16 * h);
#pragma unroll
                for (int cc = 0; cc < PF; ++cc)
#pragma unroll
                    for (int nq = 0; nq < NQ; ++nq) sacc[nq] = mfma16(kf[cc], qf[nq][c0 + cc], sacc[nq]);
                __builtin_amdgcn_sched_group_barrier(0x100, PF, 0);          // PF LDS reads
                __builtin_amdgcn_sched_group_barrier(0x008, PF * NQ, 0);     // then the MFMAs
            }
            }

            // ---- (a2) masks
            const bool need_mask = (kg + 32 > kend) || (p.causal && kg + 31 > wrow0 + coff);
            if (need_mask) {
#pragma unroll
                for (int nq = 0; nq < NQ; ++nq) {
                    const int row = wrow0 + nq * 32 + j;
                    const int lim = p.causal ? min(kend, row + 1 + coff) : kend;
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int key = kg + 8 * (i >> 2) + 4 * h + (i & 3);
                        if (key >= lim) sacc[nq][i] = -INFINITY;
                    }
                }
            }

            // ---- (a3) fold the tile into (m, S, W); exponent = s*cs - m*cs by one FMA per score
            f16x8 pb[NQ][2];
#pragma unroll
            for (int nq = 0; nq < NQ; ++nq) {
                // (no hand-written instructions on values that come straight out of an MFMA: the wait states between
                // an MFMA and the first read of its result are the compiler's to insert, and it does not look into asm)
                float ps = 0.f;
                float e[16];
                bool redo = true;
                if constexpr (LAG) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        e[i] = exp2_fast(__builtin_fmaf(sacc[nq][i], cs, nmcr[nq]));
                        if (i == 0) ps = e[0];
                        else ps += e[i];
                    }
                    redo = __builtin_amdgcn_ballot_w64(!(ps < kLagLimit)) != 0;
                }
                if (redo) {
                float mt = sacc[nq][0];
#pragma unroll
                for (int i = 1; i < 16; ++i) mt = fmaxf(mt, sacc[nq][i]);
                mt = half_max(mt);
                const float mnew = fmaxf(mrun[nq], mt);
                const float msafe = (mnew == -INFINITY) ? 0.f : mnew;      // TRIM: only the (rare) rescale uses it
                if (__builtin_amdgcn_ballot_w64(mnew > mrun[nq]) != 0) {
                    const float alpha = (mrun[nq] == -INFINITY) ? 0.f : exp2_fast((mrun[nq] - msafe) * cs);
                    srun[nq] *= alpha;
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                        for (int i = 0; i < 16; ++i) oacc[nq][mb][i] *= alpha;
                    mrun[nq] = mnew;
                }
                // -m*c; while the row has seen no key (m = -inf) a large finite value instead of +inf, so that the
                // exponent of a masked score stays -inf + finite = -inf (one minimum instead of compare + select)
                const float nmc = TRIM ? fminf(-mnew * cs, 3.0e38f) : -msafe * cs;
                if constexpr (LAG) nmcr[nq] = nmc;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    e[i] = exp2_fast(__builtin_fmaf(sacc[nq][i], cs, nmc));
                    if (TRIM && i == 0) ps = e[0];
                    else ps += e[i];
                }
                }
                srun[nq] += ps;
#pragma unroll
                for (int u = 0; u < 2; ++u)
#pragma unroll
                    for (int e2 = 0; e2 < 4; ++e2) {
                        const f32x2 pr = {e[8 * u + 2 * e2], e[8 * u + 2 * e2 + 1]};
                        const f16x2 ph = __builtin_convertvector(pr, f16x2);    // round to nearest even
                        pb[nq][u][2 * e2] = ph[0];
                        pb[nq][u][2 * e2 + 1] = ph[1];
                    }
            }

            // ---- (a4) W^T += V^T P^T.  MFMA u contracts the 16 keys held in registers 8u..8u+7 of
            // the two half-waves: element e of lane (.,h) is key 16u + 8*(e/4) + 4h + e%4.  The lane's
            // source address for the transposing read: key 4h + (lane%16)/4 (+16u, +8 for the upper four
            // elements), value columns 16*((lane/16)%2) + 4*(lane%4) .. +3 (+32 per row block).
            const unsigned char *vsrc = Vb + (kl + 4 * h + ((lane & 15) >> 2)) * VROWB +
                                        (16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2;
#pragma unroll
            for (int u = 0; u < 2; ++u) {
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    typedef short s16x4 __attribute__((ext_vector_type(4)));
                    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
                    const unsigned char *a0 = vsrc + 16 * u * VROWB + 64 * mb;
                    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(a0));
                    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(a0 + 8 * VROWB));
                    typedef short s16x8 __attribute__((ext_vector_type(8)));
                    const s16x8 both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                    const f16x8 vf = __builtin_bit_cast(f16x8, both);
#pragma unroll
                    for (int nq = 0; nq < NQ; ++nq) oacc[nq][mb] = mfma16(vf, pb[nq][u], oacc[nq][mb]);
                }
            }
        };
        if constexpr (TRIM != 0) {
#pragma unroll
            for (int ks = 0; ks < KS / 32; ++ks)
                if (ks < nact) step(ks);
        } else {
#pragma unroll 1
            for (int ks = 0; ks < nact; ++ks) step(ks);
        }
        if (t + 1 < ntiles) lstore(buf ^ 1);
        __syncthreads();
    }

    // to log2 units; per-query normaliser across the two half-waves
    float stot[NQ];
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        stot[nq] = half_sum(srun[nq]);
        mrun[nq] = (mrun[nq] == -INFINITY) ? -INFINITY : mrun[nq] * cs;
    }

    // ---- (a5) waves that split the key range merge their states through LDS
    if constexpr (WK > 1) {
        constexpr int NS = NQ * (2 + MB * 16);
        float *xs = reinterpret_cast<float *>(smem_b);
#pragma unroll
        for (int s = WK / 2; s >= 1; s >>= 1) {
            if (wk >= s && wk < 2 * s) {
                float *dst = xs + ((wk - s) * WQ + wq) * NS * 64 + lane;
                int idx = 0;
#pragma unroll
                for (int nq = 0; nq < NQ; ++nq) {
                    dst[64 * idx++] = mrun[nq];
                    dst[64 * idx++] = stot[nq];
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                        for (int i = 0; i < 16; ++i) dst[64 * idx++] = oacc[nq][mb][i];
                }
            }
            __syncthreads();
            if (wk < s) {
                const float *src = xs + (wk * WQ + wq) * NS * 64 + lane;
                int idx = 0;
#pragma unroll
                for (int nq = 0; nq < NQ; ++nq) {
                    const float mb_ = src[64 * idx++];
                    const float sb = src[64 * idx++];
                    const float mnew = fmaxf(mrun[nq], mb_);
                    const float msafe = (mnew == -INFINITY) ? 0.f : mnew;
                    const float fa = exp2_fast(mrun[nq] - msafe);
                    const float fb = exp2_fast(mb_ - msafe);
                    mrun[nq] = mnew;
                    stot[nq] = stot[nq] * fa + sb * fb;
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                        for (int i = 0; i < 16; ++i)
                            oacc[nq][mb][i] = oacc[nq][mb][i] * fa + src[64 * idx++] * fb;
                }
            }
            __syncthreads();
        }
        if (wk != 0) return;
    }

    // ---- (a7) normalise and store (FP16), or emit the block state (FP32).
    // Register 4g+t of block mb is value column 32*mb + 8g + 4h + t.
    const bool partial = p.emit_partials != 0;
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        const int row = wrow0 + nq * 32 + j;
        if (row >= n) continue;
        float f = 1.f, fold = 0.f;               // out/state = new * f + stored state * fold
        long long obase;
        if (partial) {
            const long long prow = (bh * p.num_splits + c) * (long long)n + row;
            float mo = mrun[nq], So = stot[nq];
            if (p.accumulate) {                  // stored (+) new, Eq. 3; every lane of the row reads, lane h = 0 writes
                const float ms = p.part_m[prow], Ss = p.part_S[prow];
                mo = merge_factors(mrun[nq], ms, f, fold);
                So = stot[nq] * f + Ss * fold;
            }
            if (h == 0) {
                p.part_m[prow] = p.m_natural ? mo * kLn2 : mo;
                p.part_S[prow] = So;
            }
            obase = prow * DV;
        } else {
            f = stot[nq] > 0.f ? 1.f / stot[nq] : 0.f;
            obase = out_off + (long long)row * tsv;
            if (p.lse && h == 0) p.lse[bh * (long long)n + row] = lse_of(mrun[nq], stot[nq]);
        }
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                f32x4 x = {oacc[nq][mb][4 * g] * f, oacc[nq][mb][4 * g + 1] * f, oacc[nq][mb][4 * g + 2] * f,
                           oacc[nq][mb][4 * g + 3] * f};
                const int dv = 32 * mb + 8 * g + 4 * h;
                if (partial) {
                    if (p.accumulate) x += Io<float>::load4(p.part_W, obase + dv) * fold;
                    Io<float>::store4(p.part_W, obase + dv, x);
                } else {
                    Io<_Float16>::store4(p.out, obase + dv, x);
                }
            }
    }
}

template <int D, int NQ, int WQ, int WK, int KS, int WPE, int DV = D, int TRIM = 4>
static int launch_one16(const FwdParams &p, hipStream_t s) {
    constexpr int TKB = KS * WK;
    constexpr size_t kv_bytes = (size_t)2 * (TKB * (D * 2 + 16) + TKB * (DV * 2 + 32));
    constexpr size_t xw_bytes = WK > 1 ? (size_t)(WK / 2) * WQ * NQ * (2 + DV / 2) * 64 * sizeof(float) : 0;
    constexpr size_t smem = kv_bytes > xw_bytes ? kv_bytes : xw_bytes;
    static_assert(smem <= 160 * 1024, "tile does not fit the LDS of a CU");
    // a launch that writes states for a caller keeps the exact maximum in them: the same tile without the lagging
    // reference (states of the library's own key split may carry any valid reference)
    if constexpr (TRIM >= 3) {
        if (p.emit_partials && !p.states_internal) return launch_one16<D, NQ, WQ, WK, KS, WPE, DV, (TRIM == 3 ? 2 : 1)>(p, s);
    }
    auto kern = fwd_mfma16_kernel<D, NQ, WQ, WK, KS, WPE, DV, TRIM>;
    static bool attr_done[kMaxDevices] = {};   // per instantiation and device
    if (hipError_t e = allow_dynamic_lds(kern, smem, attr_done); e != hipSuccess) return (int)e;
    const long long total = p.cu_seqlens ? (long long)p.var_tiles * p.H : (long long)p.q_tiles * p.B * p.H * p.num_splits;
    long long blocks = total;
    if (p.xcd_map == 2 && !p.cu_seqlens) blocks = (total + kNumXcd - 1) / kNumXcd * kNumXcd;
    if (blocks <= 0 || blocks > 0x7fffffffLL) return (int)hipErrorInvalidConfiguration;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(64 * WQ * WK), smem, s, p);
    return (int)hipGetLastError();
}

}  // namespace elsa
