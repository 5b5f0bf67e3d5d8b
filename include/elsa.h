/*
 * libelsa -- exact softmax attention as a reduction over the (m, S, W) monoid,
 * hand-written HIP for gfx950 (MI355X).  C ABI.
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller.  The library
 *     never allocates, frees or retains them (except the workspace registered
 *     with elsa_set_workspace, which it borrows until replaced).
 *   - Q, K, V, out are contiguous row-major [B][H][n][d] with d_v == d (elsa_attn_fwd_dv lifts
 *     that), self-attention (n queries, n keys) except for elsa_attn_fwd_cross and
 *     elsa_attn_fwd_dv.  d must be 32, 64, 96,
 *     128 or 256; 96 and 256 run on the matrix-core tiles, the one-query decode kernel and the
 *     combine only (ELSA_OPT_PATH = 1 tiles and the LDS-free small-problem tiles return
 *     ELSA_ERR_UNSUPPORTED for them).  The K (and V) slice of one (batch, head) -- one sequence of a packed batch -- must
 *     span less than 2 GiB (n*d*sizeof(element), or total_tokens*H*d*sizeof(element) for the
 *     packed layout); larger problems return ELSA_ERR_UNSUPPORTED on every path that fetches
 *     through buffer descriptors (all but the FP32 FMA tiles of ELSA_OPT_PATH = 1).
 *   - dtype: ELSA_F32 = FP32 in/out; ELSA_F16 = IEEE FP16 in/out.  Scores, the
 *     running maximum m, the normaliser S and the weighted sum W are always FP32;
 *     on the default FP16 path the exponentials are rounded to FP16 (nearest even)
 *     as operands of the PV product.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Calls
 *     only enqueue work on it; they never synchronise and never allocate.
 *     The first launch of a tile configuration on a device raises that kernel's dynamic-LDS limit
 *     with hipFuncSetAttribute (once per kernel and device), which a stream capture does not
 *     record: call an entry point once with the shapes of interest before capturing it into a HIP
 *     graph.  Work goes to the device that is current when the entry point is called.
 *   - Return ELSA_OK or an error code; nothing aborts, throws or prints.
 *     Arguments are validated before anything is launched.
 *   - Results are deterministic: no atomics; two calls on the same inputs with
 *     the same options are bit-identical.
 *   - Host threads.  Options (elsa_set_option), the lent workspace (elsa_set_workspace), the record
 *     of the last launch (elsa_last_kernel, elsa_last_splits) and the cache of the last tile choice
 *     are kept PER HOST THREAD: a new thread starts from the defaults with no workspace, and nothing
 *     one thread sets is seen by another, so threads that drive their own streams need no lock.
 *     The entry points are reentrant apart from that state.  Two calls that may run at the same time
 *     on the device (different streams) must not use the same workspace: lend one per thread.
 *   - Masks.  causal != 0: key j is visible to query i iff j <= i.  kv_len
 *     (device int32 [B], may be NULL): key j of batch b is visible iff
 *     j < kv_len[b]; values are clamped to [0, n]; query rows beyond kv_len are
 *     still computed.  A masked key is the identity element of the monoid.  A
 *     row with no visible key outputs zeros.
 */
#ifndef ELSA_H
#define ELSA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    ELSA_OK = 0,
    ELSA_ERR_INVALID_ARG = 1,  /* null pointer, B/H/n <= 0, num_splits out of range, non-finite scale */
    ELSA_ERR_UNSUPPORTED = 2,  /* d not in {32,64,96,128,256}, dtype not in {0,1}, unknown option, slice >= 2 GiB */
    ELSA_ERR_WORKSPACE = 3,    /* registered workspace too small / misaligned */
    ELSA_ERR_HIP = 4           /* the HIP runtime reported a launch failure */
};

enum { ELSA_F32 = 0, ELSA_F16 = 1 };

/*
 * y_i = sum_j e^{s_ij} v_j / sum_j e^{s_ij},  s_ij = scale * <q_i, k_j>   (Eq. 1),
 * evaluated as the reduction u_1 (+) ... (+) u_n of per-key states (s_j, 1, v_j)
 * under the merge operator of Eq. 3 and normalised by W/S (Alg. 1, last line).
 * Runs single-pass unless a workspace is registered and the problem is too small
 * to fill the GPU, in which case it splits the key range internally and combines.
 */
int elsa_attn_fwd(const void *q, const void *k, const void *v, void *out,
                  int B, int H, int n, int d, float scale, int causal,
                  int dtype, void *stream);

/* Same, with a per-batch key-padding mask kv_len (device int32 [B], NULL = none). */
int elsa_attn_fwd_masked(const void *q, const void *k, const void *v, void *out,
                         int B, int H, int n, int d, float scale, int causal,
                         const int32_t *kv_len, int dtype, void *stream);

/*
 * As elsa_attn_fwd_masked, and additionally writes the log-normaliser of every row,
 *   lse[b][h][i] = ln sum_j e^{s_ij} = m_i + ln S_i     (FP32, natural log, [B][H][n]),
 * from which the attention probabilities of the drift metrics follow as
 * P_ij = e^{s_ij - lse_i}.  A row with no visible key gets -inf.  lse must not be NULL.
 */
int elsa_attn_fwd_lse(const void *q, const void *k, const void *v, void *out, float *lse,
                      int B, int H, int n, int d, float scale, int causal,
                      const int32_t *kv_len, int dtype, void *stream);

/*
 * Rectangular attention: n_q queries against n_k keys per (batch, head) -- cross-attention,
 * chunked prefill, and decoding a few new positions against a cache.  Eq. 1 does not tie the
 * number of queries to the number of keys; every row is the same reduction over its visible keys.
 *   q, out: [B][H][n_q][d];  k, v: [B][H][n_k][d];  lse: FP32 [B][H][n_q] or NULL (not written).
 * causal != 0 aligns the LAST query with the LAST key: key j is visible to query i iff
 * j <= i + (n_k - n_q); a query with no visible key (n_k < n_q) gets zeros and lse = -inf.
 * kv_len (device int32 [B], or NULL) bounds the visible keys of a batch entry from above.
 * With a registered workspace and few query tiles the key range is split internally (up to 64
 * chunks when n_q * 8 <= n_k) and combined, which is what fills the GPU when decoding.
 * Errors as elsa_attn_fwd; additionally ELSA_ERR_INVALID_ARG for n_k <= 0.
 */
int elsa_attn_fwd_cross(const void *q, const void *k, const void *v, void *out, float *lse,
                        int B, int H, int n_q, int n_k, int d, float scale, int causal,
                        const int32_t *kv_len, int dtype, void *stream);

/*
 * Rectangular attention whose values have a width of their own: the paper's setting
 * Q, K in R^{n x d}, V in R^{n x d_v} (Sec. "Problem setup"), state (m, S, W) with W in R^{d_v};
 * the scores contract over d, the weighted sum of Eq. 1 runs over the d_v columns of V.
 *   q: [B][H][n_q][d];  k: [B][H][n_k][d];  v: [B][H][n_k][d_v];  out: [B][H][n_q][d_v];
 *   lse: FP32 [B][H][n_q] or NULL (not written).
 * Masks, causal alignment, kv_len and the internal key split exactly as elsa_attn_fwd_cross (the
 * registered workspace must hold elsa_split_kv_workspace_bytes(B, H, n_q, d_v, C) for C chunks).
 * d == d_v is forwarded to elsa_attn_fwd_cross.  Otherwise the pairs served are d, d_v in
 * {32, 64, 128} and (d, d_v) = (192, 128); they run on the matrix-core tiles (FP32 tiles for
 * ELSA_F32, FP16 tiles for ELSA_F16 with scale != 0, FP32 tiles with FP16 I/O otherwise).  Of the
 * options only ELSA_OPT_PATH in {0, 2, 3}, ELSA_OPT_VARIANT in {0, 1 = 128 query rows,
 * 3 = waves split the keys (not for FP32 tiles at d = 192)}, ELSA_OPT_SPLITS, ELSA_OPT_XCD_MAP and
 * ELSA_OPT_SNAKE apply.
 * Errors: ELSA_ERR_INVALID_ARG (NULL tensor, non-positive size, non-finite scale),
 * ELSA_ERR_UNSUPPORTED (pair, dtype or option not served; a K or V slice of 2 GiB or more),
 * ELSA_ERR_HIP (launch failure).
 */
int elsa_attn_fwd_dv(const void *q, const void *k, const void *v, void *out, float *lse,
                     int B, int H, int n_q, int n_k, int d, int d_v, float scale, int causal,
                     const int32_t *kv_len, int dtype, void *stream);

/*
 * Padding-free variable-length batches (the packed layout of the paper's
 * "padding-free variable-length" workload): Q, K, V, out are [total_tokens][H][d],
 * sequence s owns tokens cu_seqlens[s] .. cu_seqlens[s+1]-1 (device int32
 * [num_seqs+1], cu_seqlens[0] = 0, non-decreasing, last = total_tokens) and attends
 * only within itself; Eq. 1 per sequence.  No layout conversion and no padding
 * work: query tiles are cut per sequence.  max_seqlen (>= every length) only
 * guides the tile choice.  1 <= num_seqs <= 4096.  Empty sequences are allowed.
 * Offsets are clamped to [0, total_tokens] on the device; tokens not covered by any
 * sequence are left untouched in out.
 */
int elsa_attn_fwd_varlen(const void *q, const void *k, const void *v, void *out,
                         const int32_t *cu_seqlens, int num_seqs, int total_tokens, int max_seqlen,
                         int H, int d, float scale, int causal, int dtype, void *stream);

/*
 * Block states of Prop. 1.  The key range is cut into num_splits contiguous
 * chunks; chunk c covers keys [c*ceil(n/C), min(n, (c+1)*ceil(n/C))).  For every
 * query row and chunk the kernel emits the normalised state over the visible
 * keys of the chunk:
 *   part_m[b][h][c][i]    = max_j s_ij              (natural-log units)
 *   part_S[b][h][c][i]    = sum_j e^{s_ij - m}
 *   part_W[b][h][c][i][:] = sum_j e^{s_ij - m} v_j  (FP32, d values)
 * or the identity (-inf, 0, 0) when no key of the chunk is visible.
 * 1 <= num_splits <= min(n, 65535).
 */
int elsa_attn_fwd_split_kv(const void *q, const void *k, const void *v,
                           float *part_m, float *part_S, float *part_W,
                           int B, int H, int n, int d, float scale, int causal,
                           const int32_t *kv_len, int num_splits, int dtype, void *stream);

/*
 * out = W/S of part[...,0,...] (+) ... (+) part[...,C-1,...]   (Prop. 1, Eq. 3).
 * Accepts identity states; an all-identity row gives zeros.  Layouts as above.
 */
int elsa_combine(const float *part_m, const float *part_S, const float *part_W, void *out,
                 int B, int H, int n, int d, int num_splits, int dtype, void *stream);

/*
 * Streaming (memory-lean) evaluation: the keys and values arrive chunk by chunk -- a fraction of
 * the sequence at a time, e.g. staged from host memory -- and never need to be resident together.
 * The running state u = (m, S, W) of every query row lives in a caller-owned buffer; each step
 * forms the state of the new chunk and replaces u by u (+) u_chunk (Eq. 3; Prop. 1 with the
 * chunks as blocks; the identity-started sequential use of the monoid of Alg. 1, one block per
 * step).  elsa_attn_stream_finish writes y = W/S (Alg. 1, last line).
 *   state    device buffer of elsa_stream_state_bytes(B, H, n_q, d) bytes, 256-byte aligned:
 *            m [B][H][n_q] | S [B][H][n_q] | W [B][H][n_q][d], FP32, each part 256-byte aligned;
 *            m is the running maximum of scale*<q,k> in LOG2 units (times log2 e), so that
 *            re-merging adds no rounding to it.  Opaque apart from that; scale, d, dtype and the
 *            shape must stay the same over the steps of one evaluation.
 *   q        [B][H][n_q][d];  k_chunk, v_chunk: [B][H][n_chunk][d] (this step's keys only).
 *   first    != 0: the state is overwritten (no need to initialise it); 0: merged into.
 *   causal   != 0: key j OF THIS CHUNK is visible to query i iff j <= i + causal_shift.  For a
 *            chunk that starts at global key k0 of n_k keys in all, with the last query aligned
 *            to the last key, causal_shift = (n_k - n_q) - k0.  Rows that see no key of the
 *            chunk keep their state.
 *   kv_len   device int32 [B] or NULL: visible keys of this chunk per batch entry.
 * One launch per step, no key split: meant for n_q large enough to fill the GPU or for chunks
 * that arrive slower than they are consumed.  Steps of one evaluation must be ordered on the
 * stream (they read and write the state).  Errors as elsa_attn_fwd; a misaligned state returns
 * ELSA_ERR_WORKSPACE.
 */
size_t elsa_stream_state_bytes(int B, int H, int n_q, int d);
int elsa_attn_stream_step(const void *q, const void *k_chunk, const void *v_chunk, void *state,
                          int B, int H, int n_q, int n_chunk, int d, float scale,
                          int causal, int causal_shift, const int32_t *kv_len, int first,
                          int dtype, void *stream);
/* out [B][H][n_q][d] = W/S of the state; lse (FP32 [B][H][n_q], or NULL) = ln of the normaliser. */
int elsa_attn_stream_finish(const void *state, void *out, float *lse, int B, int H, int n_q, int d,
                            int dtype, void *stream);

/* Bytes of FP32 workspace that hold part_m, part_S and part_W for these sizes
 * (0 for invalid sizes).  Layout: part_m | part_S | part_W, each 256-byte aligned. */
size_t elsa_split_kv_workspace_bytes(int B, int H, int n, int d, int num_splits);

/*
 * Lend the library a device buffer (256-byte aligned) that elsa_attn_fwd[_masked]
 * may use to split the key range when B*H*ceil(n/T_q) is too small to fill the
 * GPU.  Pass (NULL, 0) to withdraw it.  The buffer belongs to the calling host thread's
 * later calls (other threads do not see it) and to the device that is current now: calls made
 * while another device is current run without it.  Calls of this thread that overlap on
 * different streams must not both use it.
 */
int elsa_set_workspace(void *dev_ptr, size_t bytes);

/*
 * For callers that cannot allocate or lend device memory (code under HIP-graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): elsa_attn_fwd_masked with the internal key split, the chunk
 * states of which live in a device array that is part of the library itself
 * (ELSA_STATIC_SCRATCH_BYTES, one copy per GPU, held until the process ends) instead of a lent
 * workspace.  Tensors, masks, dtype, stream and results as elsa_attn_fwd_masked.
 *   num_splits  0: the library chooses tile and key chunks exactly as it does for a lent workspace of
 *               that size (a single pass for problems that fill the GPU by themselves);
 *               1: single pass;  > 1: that many key chunks, ELSA_ERR_WORKSPACE if
 *               elsa_split_kv_workspace_bytes(B, H, n, d, num_splits) exceeds the array.
 * Calls nothing that allocates.  The array's device address is looked up on the first call on a device
 * (hipGetSymbolAddress), so call once before a stream capture.  All calls on one GPU share the array:
 * calls that may overlap on the device (different streams, different host threads) race on it and must
 * be ordered by the caller.  Nothing needs clearing between calls (every state read was written by the
 * same call).  Errors otherwise as elsa_attn_fwd_masked; ELSA_ERR_INVALID_ARG for num_splits < 0 or > n.
 */
#define ELSA_STATIC_SCRATCH_BYTES (64u << 20)
size_t elsa_static_scratch_bytes(void);
int elsa_attn_fwd_static(const void *q, const void *k, const void *v, void *out,
                         int B, int H, int n, int d, float scale, int causal,
                         const int32_t *kv_len, int num_splits, int dtype, void *stream);

/*
 * Measurement / tuning knobs (per host thread).  Defaults are 0.
 *   ELSA_OPT_PATH     0 = auto (FP32 I/O: FP32 MFMA; FP16 I/O: FP16 MFMA with FP32 state; one to
 *                     four queries per (batch, head), eight for FP32 at d >= 128: the FP32 vector
 *                     kernel that streams K and V),
 *                     1 = FP32 FMA (vector ALU), 2 = FP32 MFMA (FP16 inputs widened to FP32),
 *                     3 = FP16 MFMA (FP16 I/O and scale != 0 only, else ELSA_ERR_UNSUPPORTED)
 *   ELSA_OPT_VARIANT  0 = auto, otherwise a tile configuration id (see elsa_variant_name)
 *   ELSA_OPT_SPLITS   0 = auto, otherwise the number of key chunks elsa_attn_fwd uses
 *                     when a workspace is registered
 *   ELSA_OPT_XCD_MAP  block -> work order: 0 = head index fastest, key chunk slowest, longest causal
 *                     tiles of all heads first (default); 1 = query tile fastest; 2 = as 1, consecutive work
 *                     items steered to the same XCD
 *   ELSA_OPT_SNAKE    work order 0 of causal, key-padded or packed launches: 0 = longest work first
 *                     (padded batch entries by descending kv_len when 2 <= B <= 32, packed sequences
 *                     by descending length when there are at most 64) with the second run of 256
 *                     blocks walked backwards (balances the blocks that are resident together),
 *                     1 = plain order
 *   ELSA_OPT_DRY_RUN  1 = plan only: every entry point validates its arguments and chooses kernel,
 *                     tile and key chunks as usual but launches nothing and touches no tensor (no GPU
 *                     is needed); elsa_last_kernel / elsa_last_splits then report the choice
 */
enum { ELSA_OPT_PATH = 0, ELSA_OPT_VARIANT = 1, ELSA_OPT_SPLITS = 2, ELSA_OPT_XCD_MAP = 3, ELSA_OPT_SNAKE = 4,
       ELSA_OPT_DRY_RUN = 5 };
int elsa_set_option(int option, int value);
int elsa_get_option(int option, int *value);

/* Name of tile configuration `variant` for path `path` (NULL when out of range). */
const char *elsa_variant_name(int path, int variant);

/* Name of the kernel configuration the last successful forward call launched (or planned, in a dry run). */
const char *elsa_last_kernel(void);

/* Number of key chunks per (batch, head) of that call (1 = single pass, no combine launch). */
int elsa_last_splits(void);

const char *elsa_status_string(int code);

/*
 * Test hook, not part of the attention path: one wavefront reports how
 * v_mfma_f32_32x32x2_f32 lays out its result and what the half-wave exchange
 * returns, so a test can check the operand maps the forward kernel is built on.
 * out: device buffer of 5*16*64 floats.
 */
int elsa_debug_layout_probe(float *out_5x16x64, void *stream);

/*
 * Measurement hook, not part of the attention path: the issue cost of the instruction kinds the fold between the
 * two contractions is made of, alone and beside the matrix-core instructions of another wave of the same SIMD
 * (what the kernels' distance from the matrix-core roof is made of; `bench.py --issue-rates` prints the table).
 * One block per CU with waves_per_simd (1 or 2) x 4 waves; waves 0-3 issue `iters` x 16 independent instructions
 * of kind_a (iters x 8 for the MFMA kinds), waves 4-7 of kind_b.
 *   kinds: 0 v_exp_f32, 1 v_fma_f32, 2 v_add_f32, 3 v_max3_f32, 4 v_cvt_pk_f16_f32, 5 v_mfma_f32_32x32x2_f32,
 *          6 v_mfma_f32_32x32x16_f16, 7 nothing;
 *          8, 9, 10: a register-only model of one fold step of the FP16 256-row tile (two query groups per wave,
 *          d = 64, no LDS, no staging, no barrier): per iteration 8 = its 16 MFMAs alone, 9 = its fold alone (2 x
 *          (16 FMA, 16 exponentials, 16 additions, 8 conversions, the limit test)), 10 = the whole step.  A model kind
 *          runs beside itself, another model kind or kind 7 only.
 *   out: device buffer of 8 + 256 * 512 floats; out[w] = ticks of the constant 100 MHz counter that wave w of
 *        block 0 took, the rest is scratch.
 * ELSA_ERR_INVALID_ARG for a NULL buffer, an unknown kind, waves_per_simd not in {1, 2}, iters outside [1, 2^20].
 */
int elsa_debug_issue_probe(float *out, int kind_a, int kind_b, int waves_per_simd, int iters, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* ELSA_H */
