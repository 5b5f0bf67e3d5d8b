// ELSA forward, FP32 MFMA path (gfx950).
//
// One block owns T_q = 32*NQ*WQ query rows of one (batch, head) and one key
// chunk; its WQ*WK waves share K/V tiles staged in LDS.  A wave owns NQ groups of
// 32 queries and, of every tile, a slice of KS keys.  Per 32-key step it
//   1. forms the transposed score tile S^T = K Q^T with v_mfma_f32_32x32x2_f32
//      (keys are the M rows, queries the N columns), so that lane l holds 16 keys
//      of ONE query (column l%32) and lane l^32 holds the other 16;
//   2. folds the tile into the running state (m, S, W) of that query -- the merge
//      operator of Eq. 3 applied to the tile's state: in-lane max/sum over the 16
//      scores, one v_permlane32_swap across the two half-waves, rescale by
//      2^(m_old - m_new)  (scores are kept in log2 units);
//   3. accumulates W^T += V^T P^T with the same MFMA: the exponentials sit in the
//      accumulator registers exactly where the B operand of the next MFMA wants
//      them, so P never moves between lanes and never touches LDS.
// LAG = 1 (the default tiles; launches that write the output, not a state): the m of the running state may lag the
// true maximum.  (m, S, W) and (m', S 2^(m-m'), W 2^(m-m')) are the same element of the monoid and give the same W / S,
// so step 1 starts every accumulation chain from -m / NACC of the stored m -- the scores come out relative to it --
// and step 2 is exponentials and row sum only, as long as every lane's partial row sum stays below kLagLimit; otherwise
// (a row's first keys, a score far above the stored reference, a NaN) the step is redone the exact way: maximum,
// rescale, new reference.  LAG = 0 is the merge as printed in every step (tiles without the sixteen registers per
// query group that hold -m / NACC; launches that write states, whose m is the exact maximum).
// When WK > 1 the waves that split the key range merge their states through LDS
// (log2(WK) levels of the same operator).  The block then writes either
// out = W / S (Alg. 1, last line) or the state itself (Prop. 1 block state).
#pragma once
#include "elsa_common.hpp"

namespace elsa {

__device__ __forceinline__ f32x16 mfma32(float a, float b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

// D: columns of q and k (the contraction of the scores); DV: columns of v and out (rows of W^T).
template <int D, typename T, int NQ, int WQ, int WK, int KS, int WPE, int NACC, int BUFL, int DV = D, int LAG = 0>
__global__ __launch_bounds__(64 * WQ * WK, WPE) void fwd_mfma_kernel(FwdParams p) {
    constexpr int NT = 64 * WQ * WK;
    constexpr int TQ = 32 * NQ * WQ;
    constexpr int TKB = KS * WK;            // keys per LDS tile
    constexpr int KROW = D + 4;             // padded K row: 16-byte reads of 32 rows hit distinct banks
    constexpr int VROW = DV;
    constexpr int KBUF = TKB * KROW;
    constexpr int VBUF = TKB * VROW;
    constexpr int QPR = D / 4;              // 4-element groups per K row
    constexpr int QPRV = DV / 4;            // ... per V row
    constexpr int LPT = TKB * QPR / NT;     // staged groups per thread, K
    constexpr int LPTV = TKB * QPRV / NT;   // ... V
    constexpr int MB = DV / 32;             // 32-row blocks of W^T
    // Row r of block mb of W^T is value column MB*r + mb (a lane reads its MB columns of a key with
    // one LDS instruction), except for MB = 3 where it is column 32*mb + r (three 4-byte reads).
    constexpr bool VSPLIT = (MB == 3);
    constexpr bool PIN = (MB == 1 || MB == 2 || MB == 4);   // scheduling pins are written for these shapes
    static_assert(TKB * QPR % NT == 0 && TKB * QPRV % NT == 0, "tile must divide evenly over the threads");
    static_assert(D % 8 == 0 && DV % 32 == 0, "head dimensions");
    static_assert(KS % 32 == 0, "a wave consumes keys 32 at a time");
    static_assert(!LAG || NACC == 1 || NACC == 2, "the reference is split exactly over one or two chains");

    extern __shared__ __align__(16) float smem[];
    // BUFL = 2: one LDS buffer instead of two, for tiles too large to double (the next tile waits in
    // registers while the current one is consumed; two barriers per tile instead of one)
    constexpr int NBUF = BUFL == 2 ? 1 : 2;
    float *Ks = smem;                       // [NBUF][KBUF]
    float *Vs = smem + NBUF * KBUF;         // [NBUF][VBUF]

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
    const int wrow0 = q0 + wq * NQ * 32;    // first query row of this wave

    // ---- Q fragments (B operand).  MFMA step s = 4*cc + t contracts columns
    // 8*cc + t (lower half-wave) and 8*cc + 4 + t (upper); K uses the same map.
    float qf[NQ][D / 2];
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        const int row = wrow0 + nq * 32 + j;
#pragma unroll
        for (int cc = 0; cc < D / 8; ++cc) {
            f32x4 x = {0.f, 0.f, 0.f, 0.f};
            if (row < n) x = Io<T>::load4(p.q, head_off + (long long)row * ts + 8 * cc + 4 * h);
#pragma unroll
            for (int t = 0; t < 4; ++t) qf[nq][4 * cc + t] = x[t] * p.qscale;
        }
    }

    float mrun[NQ], srun[NQ];
    f32x16 oacc[NQ][MB];
    // LAG: every accumulation chain of the score MFMAs starts from -m / NACC (sixteen copies: the accumulator they add
    // to), so a step's scores come out relative to the stored reference; 0 while the row has seen no key (mrun = -inf).
    // Splitting -m over the chains keeps their partial sums as small as those of a sum started from 0 (started from
    // -m in one chain they were three times as large on average, and so was the rounding error at |m| ~ 300).
    constexpr float kLagLimit = 65536.f;
    f32x16 negm[LAG ? NQ : 1];
#pragma unroll
    for (int nq = 0; nq < (LAG ? NQ : 1); ++nq)
#pragma unroll
        for (int i = 0; i < 16; ++i) negm[nq][i] = 0.f;
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        mrun[nq] = -INFINITY;
        srun[nq] = 0.f;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int i = 0; i < 16; ++i) oacc[nq][mb][i] = 0.f;
    }

    f32x4 kst[LPT], vst[LPTV];
    // BUF: tiles are fetched through buffer descriptors whose byte range ends with the last
    // visible row of the chunk: rows beyond it read as zero, the per-thread offsets are constants
    // and the tile's position is one scalar offset -- no vector address arithmetic per tile.
    constexpr bool BUF = BUFL != 0;
    const long long slice_bytes = kend > 0 ? ((long long)(kend - 1) * ts + D) * (long long)sizeof(T) : 0;
    const __amdgpu_buffer_rsrc_t krs = make_rsrc(static_cast<const T *>(p.k) + kv_off, BUF ? slice_bytes : 0);
    const long long slice_bytes_v = kend > 0 ? ((long long)(kend - 1) * tsv + DV) * (long long)sizeof(T) : 0;
    const __amdgpu_buffer_rsrc_t vrs = make_rsrc(static_cast<const T *>(p.v) + v_off, BUF ? slice_bytes_v : 0);
    int voff[LPT], voffv[LPTV];
#pragma unroll
    for (int i = 0; i < LPT; ++i) {
        const int e = tid + i * NT;
        voff[i] = (int)(((long long)(e / QPR) * ts + 4 * (e % QPR)) * (long long)sizeof(T));
    }
#pragma unroll
    for (int i = 0; i < LPTV; ++i) {
        const int e = tid + i * NT;
        voffv[i] = (int)(((long long)(e / QPRV) * tsv + 4 * (e % QPRV)) * (long long)sizeof(T));
    }
    auto gload = [&](int t) {
        const int kb0 = kbeg + t * TKB;
        if constexpr (BUF) {
            const int soff = (int)((long long)kb0 * ts * (long long)sizeof(T));
            if constexpr (WK > 1) {
                // key-splitting tiles with a single query tile per head read K and V exactly once:
                // non-temporal loads (whole lines per instruction) keep the stream out of the caches' way
                if (p.kv_once) {
                    const int soffv = (int)((long long)kb0 * tsv * (long long)sizeof(T));
#pragma unroll
                    for (int i = 0; i < LPT; ++i) kst[i] = Io<T>::bload4_nt(krs, voff[i], soff);
#pragma unroll
                    for (int i = 0; i < LPTV; ++i) vst[i] = Io<T>::bload4_nt(vrs, voffv[i], soffv);
                    return;
                }
            }
            if constexpr (DV == D) {            // K and V loads interleaved
#pragma unroll
                for (int i = 0; i < LPT; ++i) {
                    kst[i] = Io<T>::bload4(krs, voff[i], soff);
                    vst[i] = Io<T>::bload4(vrs, voff[i], soff);
                }
            } else {
                const int soffv = (int)((long long)kb0 * tsv * (long long)sizeof(T));
#pragma unroll
                for (int i = 0; i < LPT; ++i) kst[i] = Io<T>::bload4(krs, voff[i], soff);
#pragma unroll
                for (int i = 0; i < LPTV; ++i) vst[i] = Io<T>::bload4(vrs, voffv[i], soffv);
            }
            return;
        }
#pragma unroll
        for (int i = 0; i < LPT; ++i) {
            const int e = tid + i * NT;
            const int row = e / QPR, c4 = e % QPR;
            const int key = kb0 + row;
            f32x4 kx = {0.f, 0.f, 0.f, 0.f};
            if (key < kend) kx = Io<T>::load4(p.k, kv_off + (long long)key * ts + 4 * c4);   // rows past the chunk are zero (and masked below)
            kst[i] = kx;
        }
#pragma unroll
        for (int i = 0; i < LPTV; ++i) {
            const int e = tid + i * NT;
            const int row = e / QPRV, c4 = e % QPRV;
            const int key = kb0 + row;
            f32x4 vx = {0.f, 0.f, 0.f, 0.f};
            if (key < kend) vx = Io<T>::load4(p.v, v_off + (long long)key * tsv + 4 * c4);
            vst[i] = vx;
        }
    };
    auto lstore = [&](int buf) {
#pragma unroll
        for (int i = 0; i < LPT; ++i) {
            const int e = tid + i * NT;
            const int row = e / QPR, c4 = e % QPR;
            *reinterpret_cast<f32x4 *>(&Ks[buf * KBUF + row * KROW + 4 * c4]) = kst[i];
            if constexpr (DV == D) *reinterpret_cast<f32x4 *>(&Vs[buf * VBUF + row * VROW + 4 * c4]) = vst[i];
        }
        if constexpr (DV != D) {
#pragma unroll
            for (int i = 0; i < LPTV; ++i) {
                const int e = tid + i * NT;
                const int row = e / QPRV, c4 = e % QPRV;
                *reinterpret_cast<f32x4 *>(&Vs[buf * VBUF + row * VROW + 4 * c4]) = vst[i];
            }
        }
    };

    if (ntiles > 0) {
        gload(0);
        lstore(0);
        __syncthreads();
    }
    // first key that no lane of this wave can see
    const int wave_lim = p.causal ? min(kend, wrow0 + NQ * 32 + coff) : kend;
    for (int t = 0; t < ntiles; ++t) {
        const int buf = NBUF == 2 ? (t & 1) : 0;
        if (t + 1 < ntiles) gload(t + 1);
        const float *Kb = Ks + buf * KBUF;
        const float *Vb = Vs + buf * VBUF;
        // 32-key steps of this tile in which this wave sees at least one key (wave-uniform count)
        const int kg0 = kbeg + t * TKB + wk * KS;
        const int nact = min(KS / 32, max(0, (wave_lim - kg0 + 31) / 32));
#pragma unroll 1
        for (int ks = 0; ks < nact; ++ks) {
            const int kl = wk * KS + ks * 32;           // first key of the step inside the tile
            const int kg = kg0 + ks * 32;               // its global index

            // ---- (a1) S^T = K Q^T.  NACC independent accumulation chains, summed pairwise:
            // fewer roundings at the magnitude of the full dot product.
            f32x16 sacc[NQ];
            {
                f32x16 part[NQ][NACC];
#pragma unroll
                for (int nq = 0; nq < NQ; ++nq)
#pragma unroll
                    for (int a = 0; a < NACC; ++a)
#pragma unroll
                        for (int i = 0; i < 16; ++i) part[nq][a][i] = LAG ? negm[nq][i] : 0.f;
                // K fragments are fetched one column group ahead of the MFMAs that consume them
                const float *krow = &Kb[(kl + j) * KROW + 4 * h];
                f32x4 kf = *reinterpret_cast<const f32x4 *>(krow);
#pragma unroll
                for (int cc = 0; cc < D / 8; ++cc) {
                    f32x4 kn = kf;
                    if (cc + 1 < D / 8) kn = *reinterpret_cast<const f32x4 *>(krow + 8 * (cc + 1));
                    constexpr int CPA = (D / 8) / NACC;     // column groups per chain
#pragma unroll
                    for (int tt = 0; tt < 4; ++tt)
#pragma unroll
                        for (int nq = 0; nq < NQ; ++nq)
                            part[nq][cc / CPA] = mfma32(kf[tt], qf[nq][4 * cc + tt], part[nq][cc / CPA]);
                    kf = kn;
                }
                // pin the order: two fragment reads in flight ahead of every group of MFMAs
                if constexpr (PIN) {
                    __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
#pragma unroll
                    for (int cc = 0; cc < D / 8 - 2; ++cc) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 4 * NQ, 0);
                        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                    }
                    __builtin_amdgcn_sched_group_barrier(0x008, 8 * NQ, 0);
                }
#pragma unroll
                for (int nq = 0; nq < NQ; ++nq) {
                    if constexpr (NACC == 1) sacc[nq] = part[nq][0];
                    else if constexpr (NACC == 2) sacc[nq] = part[nq][0] + part[nq][1];
                    else sacc[nq] = (part[nq][0] + part[nq][1]) + (part[nq][2] + part[nq][3]);
                }
            }

            // ---- (a2) masks: only on steps that straddle the chunk end or the diagonal
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

            // ---- (a3) fold the tile into (m, S, W): merge operator with the tile's state
#pragma unroll
            for (int nq = 0; nq < NQ; ++nq) {
                if constexpr (LAG != 0) {
                    // the scores are relative to the stored reference already: weights and their sum first; the
                    // reference is renewed only if a partial row sum passes the limit or the row has no reference yet
                    float ps = 0.f;
                    float e[16];
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        e[i] = exp2_fast(sacc[nq][i]);
                        ps += e[i];
                    }
                    const bool started = mrun[nq] != -INFINITY;
                    if (__builtin_amdgcn_ballot_w64(!(ps < kLagLimit) || !started) != 0) {
                        float mt = sacc[nq][0];
#pragma unroll
                        for (int i = 1; i < 16; ++i) mt = fmaxf(mt, sacc[nq][i]);
                        mt = half_max(mt);                   // relative to the stored reference (to 0 for a first key)
                        const bool moves = started ? (mt > 0.f) : (mt != -INFINITY);
                        const float up = moves ? mt : 0.f;
                        if (__builtin_amdgcn_ballot_w64(moves) != 0) {
                            const float alpha = started ? exp2_fast(-up) : 0.f;
                            srun[nq] *= alpha;
#pragma unroll
                            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                                for (int i = 0; i < 16; ++i) oacc[nq][mb][i] *= alpha;
                            if (moves) mrun[nq] = (started ? mrun[nq] : 0.f) + up;
                            const float nm = (mrun[nq] == -INFINITY) ? 0.f : -mrun[nq] * (1.0f / NACC);
#pragma unroll
                            for (int i = 0; i < 16; ++i) negm[nq][i] = nm;
                        }
                        ps = 0.f;
#pragma unroll
                        for (int i = 0; i < 16; ++i) {
                            e[i] = exp2_fast(sacc[nq][i] - up);
                            ps += e[i];
                        }
                    }
#pragma unroll
                    for (int i = 0; i < 16; ++i) sacc[nq][i] = e[i];
                    srun[nq] += ps;
                } else {
                float mt = sacc[nq][0];
#pragma unroll
                for (int i = 1; i < 16; ++i) mt = fmaxf(mt, sacc[nq][i]);
                mt = half_max(mt);                       // the other 16 keys of this query
                const float mnew = fmaxf(mrun[nq], mt);
                const float msafe = (mnew == -INFINITY) ? 0.f : mnew;   // identity (+) identity = identity
                // the running state is rescaled only when some row of the wave moved its maximum
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
            }

            // ---- (a4) W^T += V^T P^T.  Step i contracts keys 8g+t (lower half-wave) and
            // 8g+4+t (upper), which is where accumulator register i = 4g+t holds them.
            // Row r of block mb of W^T is value column MB*r + mb.
            if constexpr (VSPLIT) {
                const float *vcol = &Vb[(kl + 4 * h) * VROW + j];
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const float *vk = vcol + (8 * (i >> 2) + (i & 3)) * VROW;
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb) {
                        const float vx = vk[32 * mb];
#pragma unroll
                        for (int nq = 0; nq < NQ; ++nq) oacc[nq][mb] = mfma32(vx, sacc[nq][i], oacc[nq][mb]);
                    }
                }
            } else {
                typedef float vfrag __attribute__((ext_vector_type(MB)));
                const float *vcol = &Vb[(kl + 4 * h) * VROW + MB * j];
                vfrag vf = *reinterpret_cast<const vfrag *>(vcol);
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    vfrag vn = vf;                      // V fragments one key ahead of their MFMAs
                    if (i + 1 < 16)
                        vn = *reinterpret_cast<const vfrag *>(vcol + (8 * ((i + 1) >> 2) + ((i + 1) & 3)) * VROW);
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                        for (int nq = 0; nq < NQ; ++nq) oacc[nq][mb] = mfma32(vf[mb], sacc[nq][i], oacc[nq][mb]);
                    vf = vn;
                }
                if constexpr (PIN) {
                    __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
#pragma unroll
                    for (int i = 0; i < 14; ++i) {
                        __builtin_amdgcn_sched_group_barrier(0x008, MB * NQ, 0);
                        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                    }
                    __builtin_amdgcn_sched_group_barrier(0x008, 2 * MB * NQ, 0);
                }
            }
        }
        if (t + 1 < ntiles) {
            if constexpr (NBUF == 1) __syncthreads();   // every wave is done reading the only buffer
            lstore(NBUF == 2 ? (buf ^ 1) : 0);
        }
        __syncthreads();
    }

    // per-query normaliser: the two half-waves hold disjoint keys under the same maximum
    float stot[NQ];
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) stot[nq] = half_sum(srun[nq]);

    // ---- (a5) waves that split the key range merge their states through LDS
    if constexpr (WK > 1) {
        constexpr int NS = NQ * (2 + MB * 16);          // floats of state per lane
        float *xs = smem;                               // K/V tiles are dead: every wave passed the last barrier
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

    // ---- (a7) normalise and store, or emit the block state
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
        auto emit = [&](long long at, f32x4 x) {
            if (partial) {
                if (p.accumulate) x += Io<float>::load4(p.part_W, at) * fold;
                Io<float>::store4(p.part_W, at, x);
            } else {
                Io<T>::store4(p.out, at, x);
            }
        };
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            if constexpr (MB == 1) {
                const f32x4 x = {oacc[nq][0][4 * g] * f, oacc[nq][0][4 * g + 1] * f, oacc[nq][0][4 * g + 2] * f,
                                 oacc[nq][0][4 * g + 3] * f};
                emit(obase + 8 * g + 4 * h, x);
            } else if constexpr (MB == 2) {
#pragma unroll
                for (int t2 = 0; t2 < 4; t2 += 2) {
                    const f32x4 x = {oacc[nq][0][4 * g + t2] * f, oacc[nq][1][4 * g + t2] * f,
                                     oacc[nq][0][4 * g + t2 + 1] * f, oacc[nq][1][4 * g + t2 + 1] * f};
                    emit(obase + 2 * (8 * g + 4 * h + t2), x);
                }
            } else if constexpr (MB == 3) {
#pragma unroll
                for (int mb = 0; mb < 3; ++mb) {
                    const f32x4 x = {oacc[nq][mb][4 * g] * f, oacc[nq][mb][4 * g + 1] * f, oacc[nq][mb][4 * g + 2] * f,
                                     oacc[nq][mb][4 * g + 3] * f};
                    emit(obase + 32 * mb + 8 * g + 4 * h, x);
                }
            } else {
#pragma unroll
                for (int t = 0; t < 4; ++t)
#pragma unroll
                    for (int m4 = 0; m4 < MB; m4 += 4) {
                        const f32x4 x = {oacc[nq][m4][4 * g + t] * f, oacc[nq][m4 + 1][4 * g + t] * f,
                                         oacc[nq][m4 + 2][4 * g + t] * f, oacc[nq][m4 + 3][4 * g + t] * f};
                        emit(obase + MB * (8 * g + 4 * h + t) + m4, x);
                    }
            }
        }
    }
}

template <int D, typename T, int NQ, int WQ, int WK, int KS, int WPE, int NACC, int BUFL, int DV = D, int LAG = 0>
static int launch_one(const FwdParams &p, hipStream_t s) {
    // a launch that writes states for a caller keeps the exact maximum in them: the same tile without the lagging
    // reference (states of the library's own key split may carry any valid reference)
    if constexpr (LAG != 0) {
        if (p.emit_partials && !p.states_internal) return launch_one<D, T, NQ, WQ, WK, KS, WPE, NACC, BUFL, DV, 0>(p, s);
    }
    constexpr int TKB = KS * WK;
    constexpr size_t kv_bytes = (size_t)(BUFL == 2 ? 1 : 2) * (TKB * (D + 4) + TKB * DV) * sizeof(float);
    constexpr size_t xw_bytes = WK > 1 ? (size_t)(WK / 2) * WQ * NQ * (2 + DV / 2) * 64 * sizeof(float) : 0;
    constexpr size_t smem = kv_bytes > xw_bytes ? kv_bytes : xw_bytes;
    static_assert(smem <= 160 * 1024, "tile does not fit the LDS of a CU");
    auto kern = fwd_mfma_kernel<D, T, NQ, WQ, WK, KS, WPE, NACC, BUFL, DV, LAG>;
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
