// Shared device helpers for the ELSA kernels (gfx950 only).
#pragma once
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace elsa {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr int kNumXcd = 8;  // MI355X: 8 accelerator dies, blocks are dealt to them round-robin
constexpr int kNumCu = 256; // compute units

// One forward launch.  Scores are held in log2 units inside the kernels: Q is
// multiplied by qscale = scale * log2(e) once when it is loaded, so every
// exponential is a bare 2^x.
struct FwdParams {
    const void *q, *k, *v;
    void *out;                       // [B][H][n][d], used when num_splits == 1 && !emit_partials
    float *lse;                      // optional [B][H][n]: ln sum_j e^{s_ij} (dense layout, single pass)
    float *part_m, *part_S, *part_W; // [BH][C][n], [BH][C][n], [BH][C][n][d]
    const int32_t *kv_len;           // device [B] or nullptr
    int B, H, n;                     // n: queries per (batch, head)
    int nk;                          // keys per (batch, head); nk == n for self-attention
    float qscale;
    int causal;
    int num_splits;                  // C >= 1
    int chunk;                       // ceil(nk / C) keys per split
    int emit_partials;               // 1: write (m,S,W) states instead of out
    int accumulate;                  // 1 (with emit_partials, num_splits == 1, log2-unit m): merge the new state
                                     //    into the one already stored at part_m/S/W (streamed key chunks)
    int sort_batches;                // 1: dense, key padding, B <= 32, non-causal or a single query tile: batch entries in
                                     //    descending kv_len order
    int snake;                       // causal work order: 0 = plain, 1 = second run of blocks reversed (see decode_work),
                                     //    2 = also the four-run rule (kernels that keep three blocks per CU resident)
    int coff;                        // dense layout, causal: key j is visible to query i iff j <= i + coff
    int m_natural;                   // 1: part_m in natural-log units, 0: log2 units (internal)
    int states_internal;             // 1: the states written stay inside the library (internal key split): their m may be any valid reference, not the exact maximum
    int xcd_map;                     // block -> work item order, see decode_work
    int kv_once;                     // 1: one query tile per (batch, head) -- every K/V byte is read once, loads may stream
    int q_tiles;                     // ceil(n / T_q) for the launched configuration
    int tq;                          // T_q of the launched configuration
    // packed variable-length layout [total_tokens][H][d] (nullptr = dense [B][H][n][d]):
    const int32_t *cu_seqlens;       // device [num_seqs + 1], token offsets of the sequences
    int num_seqs;
    int var_tiles;                   // upper bound of query tiles over all sequences
    int total_tokens;                // offsets in cu_seqlens are clamped to [0, total_tokens]
};

struct CombineParams {
    const float *part_m, *part_S, *part_W;
    void *out;
    float *lse;                      // optional [rows]: ln of the merged normaliser
    long long rows;                  // B*H*n
    int n, num_splits;
    int m_natural;
    int f16_out;
};

__device__ __forceinline__ float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }
// ln sum_j e^{s_j} from a state with the maximum in log2 units: (m + log2 S) ln 2; -inf for the identity
__device__ __forceinline__ float lse_of(float m_log2, float S) {
    return S > 0.f ? (m_log2 + __builtin_amdgcn_logf(S)) * kLn2 : -INFINITY;
}

// The two half-waves (lanes l and l ^ 32) trade one register with v_permlane32_swap:
// afterwards r[0] holds the lower half's value and r[1] the upper half's value in
// every lane, so a symmetric reduction needs no lane test.
__device__ __forceinline__ float half_max(float x) {
    unsigned u = __float_as_uint(x);
    auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float half_sum(float x) {
    unsigned u = __float_as_uint(x);
    auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Factors of a (+) b (Eq. 3) for maxima in log2 units: a is scaled by fa, b by fb, the merged
// maximum is returned.  Two identities give (0, 0) and -inf.
__device__ __forceinline__ float merge_factors(float ma, float mb, float &fa, float &fb) {
    const float mnew = fmaxf(ma, mb);
    const float msafe = (mnew == -INFINITY) ? 0.f : mnew;
    fa = exp2_fast(ma - msafe);
    fb = exp2_fast(mb - msafe);
    return mnew;
}

// Work item (query tile, key chunk, head) of this block.  Blocks are dealt round-robin to the
// 8 XCDs, each with a private L2.
//   order 0 (default): the head index runs fastest, then the query tile, the key chunk
//     slowest.  With B*H a multiple of 8 every XCD then serves a fixed subset of heads (their
//     K and V stay in its L2), and a causal launch starts the longest query tiles of ALL heads
//     first, which is what balances the triangular work over the CUs.  (A chunk index between
//     head and tile would hand the long and the short chunk of a causal tile to fixed,
//     alternating CUs.)
//   order 1: the query tile runs fastest (consecutive blocks share a head).
//   order 2: as order 1, with consecutive work items steered to the same XCD.
struct Work {
    int qt, c;
    long long bh;
    bool valid;
    int n;             // queries of the sequence this block works on
    int nk;            // its keys
    int coff;          // causal mask: key j is visible to query i iff j <= i + coff  (coff = nk - n)
    long long base;    // element offset of query 0 of this (sequence, head) in Q and out
    long long kbase;   // element offset of key 0 in K and V
    long long ts;      // elements between consecutive tokens
};
template <int D>
__device__ __forceinline__ Work decode_work(const FwdParams &p) {
    Work r;
    if (p.cu_seqlens) {
        // packed sequences: the head index runs fastest; the tile's sequence is found by walking
        // the (short) list of sequence lengths, every value being wave-uniform
        long long w = blockIdx.x;
        // offsets are clamped so that a malformed list cannot send an access outside the tensors
        int s = 0, before = 0, len = 0, tiles = 0, beg = 0;
        if (p.num_seqs <= 64 && p.snake) {
            // Up to 64 sequences: longest first (the work of a tile grows with its sequence), ranks
            // computed across the lanes as for padded batches, and the second run of kNumCu blocks
            // walked backwards (positions beyond the last real tile stay invalid: the bound on the
            // tile count is the same for every block, so the reversal is a bijection).
            const long long bound = (long long)p.var_tiles * p.H;
            if (w >= kNumCu && w < 2 * kNumCu && w < bound) {
                const long long last = bound < 2 * kNumCu ? bound : 2 * kNumCu;
                w = kNumCu + (last - 1 - w);
            }
            const int ln = (int)(threadIdx.x & 63);
            int mybeg = 0, mylen = -1;
            if (ln < p.num_seqs) {
                mybeg = min(max(p.cu_seqlens[ln], 0), p.total_tokens);
                mylen = min(max(p.cu_seqlens[ln + 1], mybeg), p.total_tokens) - mybeg;
            }
            int rank = 0;
            for (int o = 0; o < p.num_seqs; ++o) {
                const int lo = __builtin_amdgcn_readlane(mylen, o);
                rank += (lo > mylen || (lo == mylen && o < ln)) ? 1 : 0;
            }
            const int t = (int)(w / p.H);
            int k = 0;
            for (; k < p.num_seqs; ++k) {
                const unsigned long long hit = __builtin_amdgcn_ballot_w64(ln < p.num_seqs && rank == k);
                s = hit ? __builtin_ctzll(hit) : 0;
                beg = __builtin_amdgcn_readlane(mybeg, s);
                len = __builtin_amdgcn_readlane(mylen, s);
                tiles = len > 0 ? (len + p.tq - 1) / p.tq : 0;
                if (t < before + tiles) break;
                before += tiles;
            }
            if (k >= p.num_seqs) s = p.num_seqs;
        } else {
            const int t = (int)(w / p.H);
            for (; s < p.num_seqs; ++s) {
                beg = min(max(p.cu_seqlens[s], 0), p.total_tokens);
                len = min(max(p.cu_seqlens[s + 1], beg), p.total_tokens) - beg;
                tiles = len > 0 ? (len + p.tq - 1) / p.tq : 0;
                if (t < before + tiles) break;
                before += tiles;
            }
        }
        const int hd = (int)(w % p.H);
        const int t = (int)(w / p.H);
        r.valid = s < p.num_seqs;
        r.c = 0;
        r.bh = (long long)s * p.H + hd;
        r.n = r.valid ? len : 0;
        r.nk = r.n;
        r.coff = 0;
        r.qt = t - before;
        if (p.causal) r.qt = tiles - 1 - r.qt;
        r.ts = (long long)p.H * D;
        r.base = r.valid ? (long long)beg * r.ts + (long long)hd * D : 0;
        r.kbase = r.base;
        return r;
    }
    const long long BH = (long long)p.B * p.H;
    const long long total = (long long)p.q_tiles * BH * p.num_splits;
    long long w = blockIdx.x;
    if (p.xcd_map == 2) {
        const long long per = (total + kNumXcd - 1) / kNumXcd;
        w = (w % kNumXcd) * per + w / kNumXcd;
    }
    r.valid = w < total;
    if (p.xcd_map == 0) {
        if (p.causal && p.snake && !p.sort_batches && r.valid) {
            // Longest tiles first -- but the first blocks are all resident at once, placed round-robin
            // over the CUs, with no dynamic balancing among them: the second run of kNumCu blocks is
            // walked backwards, so that the k-th longest tile shares its CU with the k-th shortest of
            // the two runs; later blocks fill slots as they free up, in descending order.  A launch of
            // exactly four runs does best with its whole second half reversed when three blocks per CU are
            // resident (the fourth block of a CU then lands where the shortest resident one finishes
            // first, and all sums are equal); with two resident blocks per CU that order would hand out
            // the last two runs shortest first (measured 5-15 % slower), so the rule is not applied there.
            if (p.snake == 2 && total > 3 * kNumCu && total <= 4 * kNumCu) {
                const long long half = total / 2;
                if (w >= half) w = half + (total - 1 - w);
            } else if (w >= kNumCu && w < 2 * kNumCu) {
                const long long last = total < 2 * kNumCu ? total : 2 * kNumCu;
                w = kNumCu + (last - 1 - w);
            }
        }
        if (p.sort_batches && r.valid) {
            // Key padding: the work of a block is set by kv_len of its batch entry.  Batch entries are
            // taken longest first (their ranks are recomputed by every block from the B lengths, B <=
            // 32), all (head, tile, chunk) items of an entry side by side, and the second run of
            // kNumCu blocks is walked backwards as for causal launches.
            if (w >= kNumCu && w < 2 * kNumCu) {
                const long long last = total < 2 * kNumCu ? total : 2 * kNumCu;
                w = kNumCu + (last - 1 - w);
            }
            const long long per_b = (long long)p.H * p.q_tiles * p.num_splits;
            const int slot = (int)(w / per_b);                  // rank of the batch entry this block serves
            const long long rem = w % per_b;
            // lane l < B holds the length of entry l and counts the entries that precede it in the
            // order (longer, or equal and earlier); the entry whose count equals the slot is ours
            const int ln = (int)(threadIdx.x & 63);
            const int mylen = ln < p.B ? min(max(p.kv_len[ln], 0), p.nk) : -1;
            int rank = 0;
            for (int o = 0; o < p.B; ++o) {
                const int lo = __builtin_amdgcn_readlane(mylen, o);
                rank += (lo > mylen || (lo == mylen && o < ln)) ? 1 : 0;
            }
            const unsigned long long hit = __builtin_amdgcn_ballot_w64(ln < p.B && rank == slot);
            const int b = hit ? __builtin_ctzll(hit) : 0;
            r.bh = (long long)b * p.H + rem % p.H;
            const long long t = rem / p.H;
            r.c = (int)(t % p.num_splits);
            r.qt = (int)(t / p.num_splits);
        } else {
            // head fastest, then the query tile, the key chunk slowest: blocks that run together work on
            // the same chunk of K and V, and the chunk index never lines up with the CU a block lands on
            // (with the chunk between head and tile, every second block of an XCD was a chunk-0 block: under a
            // causal mask the long blocks then piled up on every second CU -- 2.99 against 2.08 ms unsplit at
            // H = 8, n = 16384)
            r.bh = w % BH;
            const long long t = w / BH;
            r.qt = (int)(t % p.q_tiles);
            r.c = (int)(t / p.q_tiles);
        }
    } else {
        r.qt = (int)(w % p.q_tiles);
        const long long t = w / p.q_tiles;
        r.c = (int)(t % p.num_splits);
        r.bh = t / p.num_splits;
    }
    if (p.causal) r.qt = p.q_tiles - 1 - r.qt;   // longest rows first
    r.n = p.n;
    r.nk = p.nk;
    r.coff = p.coff;
    r.ts = D;
    r.base = r.bh * (long long)p.n * D;
    r.kbase = r.bh * (long long)p.nk * D;
    return r;
}

// Raw buffer descriptors: loads past num_records bytes return zero, so a K/V tile that sticks out
// of its chunk needs neither address arithmetic nor lane masking.
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *base, long long bytes) {
    const int nrec = bytes > 0 ? (int)(bytes < 0x7fffffffLL ? bytes : 0x7fffffffLL) : 0;
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, nrec, 0x00020000);
}

template <typename T> struct Io;
template <> struct Io<float> {
    static __device__ __forceinline__ f32x4 load4(const void *base, long long elem) {
        return *reinterpret_cast<const f32x4 *>(static_cast<const float *>(base) + elem);
    }
    static __device__ __forceinline__ void store4(void *base, long long elem, f32x4 x) {
        *reinterpret_cast<f32x4 *>(static_cast<float *>(base) + elem) = x;
    }
    static __device__ __forceinline__ f32x4 bload4(__amdgpu_buffer_rsrc_t r, int voff, int soff) {
        return __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, 0));
    }
    static __device__ __forceinline__ f32x4 bload4_nt(__amdgpu_buffer_rsrc_t r, int voff, int soff) {   // non-temporal
        return __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, 2));
    }
};
template <> struct Io<_Float16> {
    static __device__ __forceinline__ f32x4 load4(const void *base, long long elem) {
        f16x4 h = *reinterpret_cast<const f16x4 *>(static_cast<const _Float16 *>(base) + elem);
        return f32x4{(float)h[0], (float)h[1], (float)h[2], (float)h[3]};
    }
    static __device__ __forceinline__ void store4(void *base, long long elem, f32x4 x) {
        f16x4 h = {(_Float16)x[0], (_Float16)x[1], (_Float16)x[2], (_Float16)x[3]};
        *reinterpret_cast<f16x4 *>(static_cast<_Float16 *>(base) + elem) = h;
    }
    static __device__ __forceinline__ f32x4 bload4(__amdgpu_buffer_rsrc_t r, int voff, int soff) {
        const f16x4 h = __builtin_bit_cast(f16x4, __builtin_amdgcn_raw_buffer_load_b64(r, voff, soff, 0));
        return f32x4{(float)h[0], (float)h[1], (float)h[2], (float)h[3]};
    }
    static __device__ __forceinline__ f32x4 bload4_nt(__amdgpu_buffer_rsrc_t r, int voff, int soff) {
        const f16x4 h = __builtin_bit_cast(f16x4, __builtin_amdgcn_raw_buffer_load_b64(r, voff, soff, 2));
        return f32x4{(float)h[0], (float)h[1], (float)h[2], (float)h[3]};
    }
};

// Raises a kernel's dynamic-LDS limit once per device (the attribute belongs to the device's copy of the
// code object).  `done` is one flag array per kernel instantiation; setting it twice is harmless.
constexpr int kMaxDevices = 64;
template <typename Kern>
inline hipError_t allow_dynamic_lds(Kern kern, size_t bytes, bool (&done)[kMaxDevices]) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < kMaxDevices && done[dev]) return hipSuccess;
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess && dev >= 0 && dev < kMaxDevices) done[dev] = true;
    return e;
}

// Launchers implemented in the kernel translation units.  Each returns a hipError_t as int.
int launch_fwd_mfma(const FwdParams &p, int d, int f16, int variant, hipStream_t s, const char **name);
int launch_fwd_fma(const FwdParams &p, int d, int f16, int variant, hipStream_t s, const char **name);
int launch_fwd_mfma16(const FwdParams &p, int d, int variant, hipStream_t s, const char **name);
int launch_fwd_mfma_small(const FwdParams &p, int d, int f16, int nq, hipStream_t s);
int launch_fwd_decode(const FwdParams &p, int d, int f16, int nq, hipStream_t s);
// d_v != d (see elsa_fwd_dv.hip): FP32 matrix cores for either I/O type, FP16 matrix cores for FP16 I/O
int launch_fwd_dv32(const FwdParams &p, int d, int dv, int f16, int variant, hipStream_t s, const char **name);
int launch_fwd_dv16(const FwdParams &p, int d, int dv, int variant, hipStream_t s, const char **name);
int dv_variant_tq(int fp16_tiles, int variant, int d, int dv);   // queries per block (0: no such tile)
int launch_combine(const CombineParams &p, int d, hipStream_t s);
int launch_probe(float *out, hipStream_t s);
int launch_issue_probe(float *out, int kind_a, int kind_b, int waves_per_simd, int iters, hipStream_t s);
int mfma_variant_tq(int variant, int d);   // queries per block of a variant (0 if unknown)
int fma_variant_tq(int variant, int d);
int mfma16_variant_tq(int variant, int d);
const char *mfma16_variant_name(int variant);
const char *mfma_variant_name(int variant);
const char *fma_variant_name(int variant);
constexpr int kMfmaVariants = 13;
constexpr int kFmaVariants = 5;
constexpr int kMfma16Variants = 6;

}  // namespace elsa
