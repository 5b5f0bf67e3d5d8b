// C ABI of libelsa: argument checks, configuration choice, launches.  No allocation, no sync.
#include <atomic>
#include <cmath>

#include "../../include/elsa.h"
#include "elsa_common.hpp"
#include "elsa_plan.hpp"

// Scratch of elsa_attn_fwd_static: the chunk states (part_m | part_S | part_W) of one call at a time.
// Every GPU the library runs on holds its own copy of the array, at its own address, until the process
// ends.  In host code the array's name is only a handle for hipGetSymbolAddress.
static __device__ __align__(256) unsigned char scratch[ELSA_STATIC_SCRATCH_BYTES];

namespace {

// Everything a call reads besides its arguments lives here, once per HOST THREAD: a thread's options,
// the workspace it lent and the record of its last launch are its own, so threads that drive their
// own streams need no lock -- and cannot share a workspace by accident.
struct State {
    int opt[6] = {0, 0, 0, 0, 0, 0};
    void *ws = nullptr;
    size_t ws_bytes = 0;
    int ws_device = -1;              // device that was current when the workspace was lent (-1: unknown, not checked)
    const char *last = "";
    int last_splits = 1;
};
thread_local State g;

using elsa::plan::TileChoice;
using elsa::plan::choose_tiles;
using elsa::plan::choose_tiles_dv;
constexpr int kMaxSplits = elsa::plan::kMaxSplits;
static_assert(elsa::plan::kCus == elsa::kNumCu, "the planner's step times are for this part");

// The lent workspace, if this call may use it: it serves the device it was lent on only.
size_t usable_ws_bytes() {
    if (!g.ws) return 0;
    if (g.ws_device >= 0) {
        int dev = -1;
        if (hipGetDevice(&dev) != hipSuccess || dev != g.ws_device) return 0;
    }
    return g.ws_bytes;
}
int auto_splits(int B, int H, int n, int nk, int d, bool fp16_tiles, size_t ws_bytes) {
    return elsa::plan::auto_splits(g.opt[ELSA_OPT_SPLITS], B, H, n, nk, d, fp16_tiles, ws_bytes);
}
constexpr int kMaxSeqs = 4096;       // the tile -> sequence lookup walks the list linearly
using elsa::kNumCu;

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// 32, 64, 128 on every path; 96 and 256 on the matrix-core tiles, the decode kernel and the combine
bool head_dim_ok(int d) { return d == 32 || d == 64 || d == 96 || d == 128 || d == 256; }
bool head_dim_wide(int d) { return d == 96 || d == 256; }

int check_common(int B, int H, int n, int d, int dtype) {
    if (B <= 0 || H <= 0 || n <= 0) return ELSA_ERR_INVALID_ARG;
    if ((long long)B * H > 0x7fffffffLL / 64) return ELSA_ERR_INVALID_ARG;
    if (!head_dim_ok(d)) return ELSA_ERR_UNSUPPORTED;
    if (dtype != ELSA_F32 && dtype != ELSA_F16) return ELSA_ERR_UNSUPPORTED;
    return ELSA_OK;
}

// paths: 1 = FP32 vector FMA, 2 = FP32 MFMA, 3 = FP16 MFMA (FP16 I/O only)
int variant_count(int path) {
    return path == 1 ? elsa::kFmaVariants : path == 3 ? elsa::kMfma16Variants : elsa::kMfmaVariants;
}
int variant_tq(int path, int variant, int d) {
    return path == 1 ? elsa::fma_variant_tq(variant, d)
         : path == 3 ? elsa::mfma16_variant_tq(variant, d) : elsa::mfma_variant_tq(variant, d);
}

// Tile configuration when the caller did not force one (FP32 MFMA ids in brackets).  Measured on
// MI355X: the 128-row tile with 32-key LDS tiles [7] keeps three waves per SIMD resident and is
// within 2 % of the fastest configuration at every size while using two score chains; d = 128
// uses the 128-row tile [1]; when fewer than 192 such blocks exist, the configuration whose waves
// split the key range [3].  The 256-row tiles [2, 4] are opt-in.
int pick_variant(int path, long long BH, int n, int nk, int d, int splits, int causal) {
    if (g.opt[ELSA_OPT_VARIANT] >= 1 && g.opt[ELSA_OPT_VARIANT] <= variant_count(path)) return g.opt[ELSA_OPT_VARIANT];
    // one query tile against a long key range: the waves of a block split the keys, not the queries
    // (FP32, d = 128, up to 32 queries: four key waves on a single-buffered 128-key tile, so that no wave idles)
    if (path == 2 && d == 128 && (long long)n * 8 <= nk && n <= 32) return 12;
    if (path != 1 && (long long)n * 8 <= nk && n <= variant_tq(path, 3, d)) return 3;
    if (path == 1) {
        const long long blocks = BH * ((n + 255) / 256) * splits;
        return blocks >= kNumCu ? 1 : 2;
    }
    const long long b256 = BH * ((n + 255) / 256) * splits;
    const long long b128 = BH * ((n + 127) / 128) * splits;
    // FP16, d <= 64: the 256-row tile (two blocks per CU) wins from 512 such blocks up when they fill the 512 places
    // evenly (640 blocks = 1.25 rounds: 0.92-0.96 of the 128-row tile's speed; 512 / 1024 / 1280 / 2560: 1.02-1.10); under a
    // causal mask its diagonal tiles waste twice as much, which pays off only on long sequences with many blocks
    // (n >= 16384 and 1024 blocks: 1.04-1.07; n = 8192 or 512 blocks: 0.83-0.98)
    if (path == 3) {
        if (d <= 64 && n >= 256) {
            const long long places = 2 * kNumCu, rounds = (b256 + places - 1) / places;
            if (!causal && b256 >= places && 100 * b256 >= 80 * rounds * places) return 2;
            if (causal && n >= 16384 && b256 >= 4 * kNumCu) return 2;
        }
        return b128 >= (3 * kNumCu) / 4 ? 1 : 3;
    }
    if (b128 < (3 * kNumCu) / 4) return 3;
    return d <= 64 ? 7 : 1;
}

// The LDS-free one-wave-per-tile kernel serves dense single-pass calls only.
bool small_kernel_ok(const int32_t *cu_seqlens, int splits, int emit, int n, int nk) {
    return !cu_seqlens && splits == 1 && !emit && n == nk;
}

// Optional parts of a forward launch.
struct Extra {
    const int32_t *cu_seqlens = nullptr;         // packed layout
    int num_seqs = 0, total_tokens = 0;
    float *lse = nullptr;
    int nk = 0;                                  // keys per (batch, head); 0 = as many as queries
    int accumulate = 0;                          // merge the emitted state into the stored one
    bool has_coff = false;                       // causal diagonal given explicitly (streamed chunks)
    int coff = 0;
    int variant = 0;                             // matrix-core tile chosen by the caller (0: pick_variant decides)
    bool states_internal = false;                // the states written are consumed by the library's own combine pass only
};

int run_forward(const void *q, const void *k, const void *v, void *out, float *pm, float *pS, float *pW,
                int B, int H, int n, int d, float scale, int causal, const int32_t *kv_len,
                int num_splits, int emit, int m_natural, int dtype, void *stream, const Extra &x = Extra()) {
    const int32_t *cu_seqlens = x.cu_seqlens;
    const int num_seqs = x.num_seqs, total_tokens = x.total_tokens;
    float *lse = x.lse;
    const int nk = x.nk > 0 ? x.nk : n;          // self-attention: as many keys as queries
    // auto: FP32 I/O -> FP32 MFMA; FP16 I/O -> FP16 MFMA (needs a non-zero scale)
    int path = g.opt[ELSA_OPT_PATH];
    if (path == 0) path = (dtype == ELSA_F16 && scale != 0.f) ? 3 : 2;
    if (path == 3 && (dtype != ELSA_F16 || scale == 0.f)) return ELSA_ERR_UNSUPPORTED;
    // one to four queries per (batch, head): the vector kernel that streams K and V once
    int decode_variant = 0;
    // (up to eight for FP32 at d >= 128, where the key-splitting matrix-core tile keeps only half
    // of its waves busy: 0.89 against 0.99 ms at n_q = 8, n_k = 32768, B*H = 80)
    const int decode_max = (dtype == ELSA_F32 && d >= 128) ? 8 : 4;
    if (g.opt[ELSA_OPT_PATH] == 0 && g.opt[ELSA_OPT_VARIANT] == 0 && !cu_seqlens && n <= decode_max) {
        path = 1;
        decode_variant = (n == 1 || head_dim_wide(d)) ? 3 : 4;
        if (n > 4 && dtype == ELSA_F32 && d == 128) decode_variant = 5;   // eight queries per block: K and V read once
    }
    if (path == 1 && g.opt[ELSA_OPT_VARIANT] >= 3 && g.opt[ELSA_OPT_VARIANT] <= 5) {
        if (cu_seqlens) return ELSA_ERR_UNSUPPORTED;
        if (g.opt[ELSA_OPT_VARIANT] == 5 && (dtype != ELSA_F32 || d != 128)) return ELSA_ERR_UNSUPPORTED;
        decode_variant = g.opt[ELSA_OPT_VARIANT];
    }
    if (head_dim_wide(d)) {                      // no FMA tiles, no four-query decode, no LDS-free tiles
        if (path == 1 && decode_variant != 3) return ELSA_ERR_UNSUPPORTED;
        if (path == 2 && (g.opt[ELSA_OPT_VARIANT] == 9 || g.opt[ELSA_OPT_VARIANT] == 10)) return ELSA_ERR_UNSUPPORTED;
    }
    // the K/V slice of one (sequence, head) is addressed through a 31-bit buffer range
    const long long tok_stride = cu_seqlens ? (long long)H * d : d;
    const long long longest = cu_seqlens ? total_tokens : (nk > n ? nk : n);
    if ((path != 1 || decode_variant) && longest * tok_stride * (dtype == ELSA_F16 ? 2 : 4) >= 0x7fffffffLL) return ELSA_ERR_UNSUPPORTED;
    int variant = decode_variant ? decode_variant : pick_variant(path, (long long)B * H, n, nk, d, num_splits, causal);
    const bool hinted = (path == 2 || path == 3) && !decode_variant && x.variant > 0 && g.opt[ELSA_OPT_VARIANT] == 0;
    if (hinted) variant = x.variant;
    if (path == 2 && !hinted) {
        const bool ok = small_kernel_ok(cu_seqlens, num_splits, emit, n, nk);
        // thousands of tiny problems (window attention); at n = 128 or d = 128 the 128-row tile is faster
        if (g.opt[ELSA_OPT_VARIANT] == 0 && ok && d <= 64 && n <= 96 && (long long)B * H * ((n + 31) / 32) >= 4 * kNumCu)
            variant = 10;
        if ((variant == 9 || variant == 10) && !ok) variant = d <= 64 ? 7 : 1;
    }
    const int tq = variant_tq(path, variant, d);
    if (tq <= 0) return ELSA_ERR_UNSUPPORTED;
    elsa::FwdParams p{};
    p.q = q; p.k = k; p.v = v; p.out = out;
    p.lse = lse;
    p.part_m = pm; p.part_S = pS; p.part_W = pW;
    p.kv_len = kv_len;
    p.B = B; p.H = H; p.n = n; p.nk = nk;
    p.qscale = scale * elsa::kLog2e;
    p.causal = causal ? 1 : 0;
    p.num_splits = num_splits;
    p.chunk = (nk + num_splits - 1) / num_splits;
    p.emit_partials = emit;
    p.accumulate = x.accumulate;
    p.coff = x.has_coff ? x.coff : nk - n;       // last query aligned with the last key
    p.m_natural = m_natural;
    p.states_internal = (emit && x.states_internal && !x.accumulate && !m_natural) ? 1 : 0;
    p.q_tiles = (n + tq - 1) / tq;
    p.tq = tq;
    p.kv_once = p.q_tiles == 1 ? 1 : 0;
    p.cu_seqlens = cu_seqlens;
    p.num_seqs = num_seqs;
    p.total_tokens = total_tokens;
    // every sequence wastes at most one partly filled tile
    p.var_tiles = cu_seqlens ? (int)(((long long)total_tokens + tq - 1) / tq + num_seqs) : 0;
    p.xcd_map = g.opt[ELSA_OPT_XCD_MAP];
    // FP16 tiles on a K/V set beyond the 256 MB of last-level cache (>= 320 MB, thousands of blocks, heads a multiple of the
    // 8 XCDs): consecutive query tiles of one head per XCD, so that the 64 resident blocks of an XCD
    // share one K/V stream (LLaMA-13B shape at 32K: 12.6 -> 11.7 ms causal, 25.7 -> 23.1 ms non-causal;
    // smaller launches lose more to the coarser balance than they gain, the FP32 tiles gain nothing)
    if (p.xcd_map == 0 && path == 3 && !cu_seqlens && ((long long)B * H) % elsa::kNumXcd == 0 &&
        4.0 * B * H * nk * d >= 320.0 * 1048576.0 && (long long)p.q_tiles * B * H * num_splits >= 16 * kNumCu)
        p.xcd_map = 2;
    p.snake = g.opt[ELSA_OPT_SNAKE] == 1 ? 0 : 1;
    if (p.snake && path == 2 && variant == 7 && d <= 64) p.snake = 2;   // three resident blocks per CU: four-run rule
    p.sort_batches = (kv_len && !cu_seqlens && (!causal || p.q_tiles == 1) && B >= 2 && B <= 32 && p.snake && p.xcd_map == 0) ? 1 : 0;
    const long long total = (long long)p.q_tiles * B * H * num_splits;
    if (total > 0x7fffffffLL - 8) return ELSA_ERR_INVALID_ARG;
    g.last_splits = num_splits;
    if (g.opt[ELSA_OPT_DRY_RUN]) {               // plan only: report what would be launched
        const char *planned = path == 1 ? elsa::fma_variant_name(variant)
                            : path == 3 ? elsa::mfma16_variant_name(variant) : elsa::mfma_variant_name(variant);
        g.last = planned ? planned : "";
        return ELSA_OK;
    }
    const char *name = nullptr;
    const hipStream_t s = static_cast<hipStream_t>(stream);
    const int rc = path == 1   ? elsa::launch_fwd_fma(p, d, dtype == ELSA_F16, variant, s, &name)
                   : path == 3 ? elsa::launch_fwd_mfma16(p, d, variant, s, &name)
                               : elsa::launch_fwd_mfma(p, d, dtype == ELSA_F16, variant, s, &name);
    if (rc != 0) return ELSA_ERR_HIP;
    g.last = name ? name : "";
    return ELSA_OK;
}

// (d, d_v) pairs with d_v != d: the matrix-core tiles only (no vector-FMA, decode or LDS-free kernels)
bool dv_pair_ok(int d, int dv) {
    if (d == dv) return false;
    if (d == 192) return dv == 128;
    return (d == 32 || d == 64 || d == 128) && (dv == 32 || dv == 64 || dv == 128);
}

// Forward launch for d_v != d; dense layout only.  Tile 3 (the waves of a block split the keys) for a
// single query tile against a long key range or when the 128-row tile yields too few blocks, tile 1
// (128 query rows) otherwise.
int run_forward_dv(const void *q, const void *k, const void *v, void *out, float *lse, float *pm, float *pS, float *pW,
                   int B, int H, int n, int nk, int d, int dv, float scale, int causal, const int32_t *kv_len,
                   int num_splits, int emit, int dtype, void *stream, int chosen_variant = 0) {
    int path = g.opt[ELSA_OPT_PATH];
    if (path == 0) path = (dtype == ELSA_F16 && scale != 0.f) ? 3 : 2;
    if (path == 1) return ELSA_ERR_UNSUPPORTED;
    if (path == 3 && (dtype != ELSA_F16 || scale == 0.f)) return ELSA_ERR_UNSUPPORTED;
    const int fp16_tiles = path == 3;
    const long long esz = dtype == ELSA_F16 ? 2 : 4;
    if ((long long)(nk > n ? nk : n) * (d > dv ? d : dv) * esz >= 0x7fffffffLL) return ELSA_ERR_UNSUPPORTED;
    int variant = g.opt[ELSA_OPT_VARIANT];
    if (variant != 0 && variant != 1 && variant != 3 && variant != 6) return ELSA_ERR_UNSUPPORTED;
    const int tq3 = elsa::dv_variant_tq(fp16_tiles, 3, d, dv);
    if (variant == 0 && chosen_variant != 0) variant = chosen_variant;    // from the block-placement model
    // FP16 tiles with a 128-wide (or wider) operand: the 256-row tile of eight query waves where its blocks fill the CUs
    // evenly (the rule measured at d_v = d = 128)
    if (g.opt[ELSA_OPT_VARIANT] == 0 && fp16_tiles && !emit && num_splits == 1 && (long long)n * 8 > nk &&
        elsa::dv_variant_tq(1, 6, d, dv) > 0 && elsa::plan::wide_fp16_tile_pays((long long)B * H, n, 128, causal))
        variant = 6;
    if (variant == 0) {
        const long long b128 = (long long)B * H * ((n + 127) / 128) * num_splits;
        variant = 1;
        if (tq3 > 0 && (((long long)n * 8 <= nk && n <= tq3) || b128 < (3 * kNumCu) / 4)) variant = 3;
    }
    const int tq = elsa::dv_variant_tq(fp16_tiles, variant, d, dv);
    if (tq <= 0) return ELSA_ERR_UNSUPPORTED;
    elsa::FwdParams p{};
    p.q = q; p.k = k; p.v = v; p.out = out;
    p.lse = lse;
    p.part_m = pm; p.part_S = pS; p.part_W = pW;
    p.kv_len = kv_len;
    p.B = B; p.H = H; p.n = n; p.nk = nk;
    p.qscale = scale * elsa::kLog2e;
    p.causal = causal ? 1 : 0;
    p.num_splits = num_splits;
    p.chunk = (nk + num_splits - 1) / num_splits;
    p.emit_partials = emit;
    p.coff = nk - n;                             // last query aligned with the last key
    p.q_tiles = (n + tq - 1) / tq;
    p.tq = tq;
    p.kv_once = p.q_tiles == 1 ? 1 : 0;
    p.xcd_map = g.opt[ELSA_OPT_XCD_MAP];
    p.snake = g.opt[ELSA_OPT_SNAKE] == 1 ? 0 : 1;
    p.sort_batches = (kv_len && (!causal || p.q_tiles == 1) && B >= 2 && B <= 32 && p.snake && p.xcd_map == 0) ? 1 : 0;
    if ((long long)p.q_tiles * B * H * num_splits > 0x7fffffffLL - 8) return ELSA_ERR_INVALID_ARG;
    g.last_splits = num_splits;
    if (g.opt[ELSA_OPT_DRY_RUN]) {
        g.last = fp16_tiles ? (variant == 3 ? "mfma16_dv_xwave" : "mfma16_dv_q128") : (variant == 3 ? "mfma_dv_xwave" : "mfma_dv_q128");
        return ELSA_OK;
    }
    const char *name = nullptr;
    const hipStream_t s = static_cast<hipStream_t>(stream);
    const int rc = fp16_tiles ? elsa::launch_fwd_dv16(p, d, dv, variant, s, &name)
                              : elsa::launch_fwd_dv32(p, d, dv, dtype == ELSA_F16, variant, s, &name);
    if (rc != 0) return ELSA_ERR_HIP;
    g.last = name ? name : "";
    return ELSA_OK;
}

void carve(void *ws, int B, int H, int n, int d, int C, float **pm, float **pS, float **pW) {
    const size_t rows = (size_t)B * H * C * n;
    char *base = static_cast<char *>(ws);
    *pm = reinterpret_cast<float *>(base);
    *pS = reinterpret_cast<float *>(base + align256(rows * 4));
    *pW = reinterpret_cast<float *>(base + 2 * align256(rows * 4));
    (void)d;
}

// ---- the static scratch array (declared at file scope above): its address is looked up once per device,
// with that device current, and kept; kernels and copies take that address, never the array's name.
std::atomic<void *> scratch_ptr[elsa::kMaxDevices];    // zero-initialised; a lost race stores the same address twice

int static_scratch(void **ptr) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= elsa::kMaxDevices) {
        (void)hipGetLastError();
        return ELSA_ERR_HIP;
    }
    void *p = scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return ELSA_ERR_HIP;
        }
        scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *ptr = p;
    return ELSA_OK;
}

}  // namespace

extern "C" {

size_t elsa_split_kv_workspace_bytes(int B, int H, int n, int d, int num_splits) {
    return elsa::plan::workspace_bytes(B, H, n, d, num_splits);
}

int elsa_set_workspace(void *dev_ptr, size_t bytes) {
    if ((dev_ptr == nullptr) != (bytes == 0)) return ELSA_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(dev_ptr) & 255) return ELSA_ERR_WORKSPACE;
    g.ws = dev_ptr;
    g.ws_bytes = bytes;
    g.ws_device = -1;
    if (dev_ptr) {                               // no GPU (a dry-run plan on a CPU machine): left unknown
        int dev = -1;
        if (hipGetDevice(&dev) == hipSuccess) g.ws_device = dev;
        else (void)hipGetLastError();
    }
    return ELSA_OK;
}

// The whole path for one dense problem.  `ws` / `ws_bytes`: device memory this call may keep chunk
// states in (the workspace the thread lent, or the library's static scratch array); `force_splits`
// > 0 fixes the number of key chunks (the caller has checked that their states fit).
static int attn_fwd_impl(const void *q, const void *k, const void *v, void *out, float *lse,
                         int B, int H, int n, int d, float scale, int causal,
                         const int32_t *kv_len, int dtype, void *stream, int nk,
                         void *ws, size_t ws_bytes, int force_splits = 0) {
    if (!q || !k || !v || !out) return ELSA_ERR_INVALID_ARG;
    if (!std::isfinite(scale)) return ELSA_ERR_INVALID_ARG;
    if (nk <= 0) nk = n;
    int rc = check_common(B, H, n, d, dtype);
    if (rc != ELSA_OK) return rc;
    const bool fp16_tiles = dtype == ELSA_F16 && scale != 0.f && (g.opt[ELSA_OPT_PATH] == 0 || g.opt[ELSA_OPT_PATH] == 3);
    int C = force_splits > 0 ? force_splits : (ws ? auto_splits(B, H, n, nk, d, fp16_tiles, ws_bytes) : 1);
    Extra x;
    x.nk = nk;
    // small problems: tile shape and key chunks together, from the block-placement model
    const long long b128 = (long long)B * H * ((n + 127) / 128);
    const bool fp32_tiles = !fp16_tiles && (g.opt[ELSA_OPT_PATH] == 0 || g.opt[ELSA_OPT_PATH] == 2);
    const bool window = !fp16_tiles && n <= 96 && (long long)B * H * ((n + 31) / 32) >= 4 * kNumCu;   // served by the LDS-free tile
    const bool modelled = fp32_tiles || fp16_tiles;
    if (modelled && force_splits <= 0 && g.opt[ELSA_OPT_VARIANT] == 0 && g.opt[ELSA_OPT_SPLITS] == 0 && b128 <= 12 * kNumCu &&
        (long long)n * 8 > nk && n > 8 && n <= 16384 && !window) {
        int max_c = 1;
        if (ws && !fp16_tiles) {                  // the FP16 tiles are not cut outside decoding
            max_c = 4;                           // more chunks were never the best measured choice outside decoding
            while (max_c > 1 && elsa_split_kv_workspace_bytes(B, H, n, d, max_c) > ws_bytes) --max_c;
        }
        const TileChoice tc = choose_tiles(fp16_tiles, (long long)B * H, n, nk, d, causal, max_c);
        x.variant = tc.variant;
        C = tc.splits;
    }
    // FP16 tiles at d >= 96: the 256-row tile of eight query waves where its coarser blocks still fill the CUs
    if (fp16_tiles && C == 1 && g.opt[ELSA_OPT_VARIANT] == 0 && (long long)n * 8 > nk &&
        elsa::plan::wide_fp16_tile_pays((long long)B * H, n, d, causal))
        x.variant = 6;
    if (C == 1) {
        x.lse = lse;
        return run_forward(q, k, v, out, nullptr, nullptr, nullptr, B, H, n, d, scale, causal, kv_len, 1, 0, 0, dtype,
                           stream, x);
    }
    float *pm, *pS, *pW;
    carve(ws, B, H, n, d, C, &pm, &pS, &pW);
    // internal split: maxima stay in log2 units, so the second pass adds no rounding of m; the states never leave the
    // library, so the tiles may keep their lagging reference in them
    x.states_internal = true;
    rc = run_forward(q, k, v, nullptr, pm, pS, pW, B, H, n, d, scale, causal, kv_len, C, 1, 0, dtype, stream, x);
    if (rc != ELSA_OK) return rc;
    if (g.opt[ELSA_OPT_DRY_RUN]) return ELSA_OK;
    elsa::CombineParams cp{pm, pS, pW, out, lse, (long long)B * H * n, n, C, 0, dtype == ELSA_F16};
    return elsa::launch_combine(cp, d, static_cast<hipStream_t>(stream)) == 0 ? ELSA_OK : ELSA_ERR_HIP;
}

int elsa_attn_fwd_masked(const void *q, const void *k, const void *v, void *out,
                         int B, int H, int n, int d, float scale, int causal,
                         const int32_t *kv_len, int dtype, void *stream) {
    const size_t wb = usable_ws_bytes();
    return attn_fwd_impl(q, k, v, out, nullptr, B, H, n, d, scale, causal, kv_len, dtype, stream, 0, wb ? g.ws : nullptr, wb);
}

size_t elsa_static_scratch_bytes(void) { return (size_t)ELSA_STATIC_SCRATCH_BYTES; }

int elsa_attn_fwd_static(const void *q, const void *k, const void *v, void *out,
                         int B, int H, int n, int d, float scale, int causal,
                         const int32_t *kv_len, int num_splits, int dtype, void *stream) {
    if (!q || !k || !v || !out) return ELSA_ERR_INVALID_ARG;
    if (!std::isfinite(scale)) return ELSA_ERR_INVALID_ARG;
    const int rc = check_common(B, H, n, d, dtype);
    if (rc != ELSA_OK) return rc;
    if (num_splits < 0 || num_splits > n || num_splits > kMaxSplits) return ELSA_ERR_INVALID_ARG;
    // a requested chunk count whose states do not fit the array is an error, never a silent fallback
    if (num_splits > 1 && elsa_split_kv_workspace_bytes(B, H, n, d, num_splits) > (size_t)ELSA_STATIC_SCRATCH_BYTES)
        return ELSA_ERR_WORKSPACE;
    void *ws = nullptr;
    if (g.opt[ELSA_OPT_DRY_RUN]) ws = reinterpret_cast<void *>(256);    // a plan touches no memory
    else if (const int e = static_scratch(&ws); e != ELSA_OK) return e;
    // Nothing in the array has to start at zero: the first pass writes the state of every (row, chunk),
    // the identity for chunks that a mask empties, before the combine pass reads it.
    return attn_fwd_impl(q, k, v, out, nullptr, B, H, n, d, scale, causal, kv_len, dtype, stream, 0, ws,
                         (size_t)ELSA_STATIC_SCRATCH_BYTES, num_splits);
}

int elsa_attn_fwd_lse(const void *q, const void *k, const void *v, void *out, float *lse,
                      int B, int H, int n, int d, float scale, int causal,
                      const int32_t *kv_len, int dtype, void *stream) {
    if (!lse) return ELSA_ERR_INVALID_ARG;
    const size_t wb = usable_ws_bytes();
    return attn_fwd_impl(q, k, v, out, lse, B, H, n, d, scale, causal, kv_len, dtype, stream, 0, wb ? g.ws : nullptr, wb);
}

int elsa_attn_fwd_cross(const void *q, const void *k, const void *v, void *out, float *lse,
                        int B, int H, int n_q, int n_k, int d, float scale, int causal,
                        const int32_t *kv_len, int dtype, void *stream) {
    if (n_k <= 0) return ELSA_ERR_INVALID_ARG;
    const size_t wb = usable_ws_bytes();
    return attn_fwd_impl(q, k, v, out, lse, B, H, n_q, d, scale, causal, kv_len, dtype, stream, n_k, wb ? g.ws : nullptr, wb);
}

int elsa_attn_fwd_dv(const void *q, const void *k, const void *v, void *out, float *lse,
                     int B, int H, int n_q, int n_k, int d, int d_v, float scale, int causal,
                     const int32_t *kv_len, int dtype, void *stream) {
    if (n_k <= 0) return ELSA_ERR_INVALID_ARG;
    const size_t wb = usable_ws_bytes();
    void *const ws = wb ? g.ws : nullptr;
    if (d == d_v) return attn_fwd_impl(q, k, v, out, lse, B, H, n_q, d, scale, causal, kv_len, dtype, stream, n_k, ws, wb);
    if (!q || !k || !v || !out) return ELSA_ERR_INVALID_ARG;
    if (!std::isfinite(scale)) return ELSA_ERR_INVALID_ARG;
    if (B <= 0 || H <= 0 || n_q <= 0) return ELSA_ERR_INVALID_ARG;
    if ((long long)B * H > 0x7fffffffLL / 64) return ELSA_ERR_INVALID_ARG;
    if (dtype != ELSA_F32 && dtype != ELSA_F16) return ELSA_ERR_UNSUPPORTED;
    if (!dv_pair_ok(d, d_v)) return ELSA_ERR_UNSUPPORTED;
    const bool fp16_tiles = dtype == ELSA_F16 && scale != 0.f && (g.opt[ELSA_OPT_PATH] == 0 || g.opt[ELSA_OPT_PATH] == 3);
    // the states of a key split hold d_v columns: the workspace is sized by d_v
    int C = ws ? auto_splits(B, H, n_q, n_k, d_v, fp16_tiles, wb) : 1;
    // small problems: tile shape and key chunks together, from the block-placement model (as for d_v = d)
    int chosen = 0;
    const long long b128 = (long long)B * H * ((n_q + 127) / 128);
    const bool tiles_free = g.opt[ELSA_OPT_PATH] == 0 || (g.opt[ELSA_OPT_PATH] == 3 && fp16_tiles) || (g.opt[ELSA_OPT_PATH] == 2 && !fp16_tiles);
    if (tiles_free && g.opt[ELSA_OPT_VARIANT] == 0 && g.opt[ELSA_OPT_SPLITS] == 0 && b128 <= 12 * kNumCu &&
        (long long)n_q * 8 > n_k && n_q > 8 && n_q <= 16384) {
        int max_c = 1;
        if (ws && !fp16_tiles) {                  // the FP16 tiles are not cut outside decoding
            max_c = 4;
            while (max_c > 1 && elsa_split_kv_workspace_bytes(B, H, n_q, d_v, max_c) > wb) --max_c;
        }
        const TileChoice tc = choose_tiles_dv(fp16_tiles, (long long)B * H, n_q, n_k, d, d_v, causal, max_c);
        chosen = tc.variant;
        C = tc.splits;
    }
    if (C == 1)
        return run_forward_dv(q, k, v, out, lse, nullptr, nullptr, nullptr, B, H, n_q, n_k, d, d_v, scale, causal, kv_len,
                              1, 0, dtype, stream, chosen);
    float *pm, *pS, *pW;
    carve(ws, B, H, n_q, d_v, C, &pm, &pS, &pW);
    const int rc = run_forward_dv(q, k, v, nullptr, nullptr, pm, pS, pW, B, H, n_q, n_k, d, d_v, scale, causal, kv_len,
                                  C, 1, dtype, stream, chosen);
    if (rc != ELSA_OK) return rc;
    if (g.opt[ELSA_OPT_DRY_RUN]) return ELSA_OK;
    elsa::CombineParams cp{pm, pS, pW, out, lse, (long long)B * H * n_q, n_q, C, 0, dtype == ELSA_F16};
    return elsa::launch_combine(cp, d_v, static_cast<hipStream_t>(stream)) == 0 ? ELSA_OK : ELSA_ERR_HIP;
}

int elsa_attn_fwd(const void *q, const void *k, const void *v, void *out,
                  int B, int H, int n, int d, float scale, int causal, int dtype, void *stream) {
    return elsa_attn_fwd_masked(q, k, v, out, B, H, n, d, scale, causal, nullptr, dtype, stream);
}

int elsa_attn_fwd_split_kv(const void *q, const void *k, const void *v,
                           float *part_m, float *part_S, float *part_W,
                           int B, int H, int n, int d, float scale, int causal,
                           const int32_t *kv_len, int num_splits, int dtype, void *stream) {
    if (!q || !k || !v || !part_m || !part_S || !part_W) return ELSA_ERR_INVALID_ARG;
    if (!std::isfinite(scale)) return ELSA_ERR_INVALID_ARG;
    int rc = check_common(B, H, n, d, dtype);
    if (rc != ELSA_OK) return rc;
    if (num_splits < 1 || num_splits > n || num_splits > kMaxSplits) return ELSA_ERR_INVALID_ARG;
    return run_forward(q, k, v, nullptr, part_m, part_S, part_W, B, H, n, d, scale, causal, kv_len, num_splits, 1, 1,
                       dtype, stream);
}

int elsa_combine(const float *part_m, const float *part_S, const float *part_W, void *out,
                 int B, int H, int n, int d, int num_splits, int dtype, void *stream) {
    if (!part_m || !part_S || !part_W || !out) return ELSA_ERR_INVALID_ARG;
    int rc = check_common(B, H, n, d, dtype);
    if (rc != ELSA_OK) return rc;
    if (num_splits < 1 || num_splits > n || num_splits > kMaxSplits) return ELSA_ERR_INVALID_ARG;
    if (g.opt[ELSA_OPT_DRY_RUN]) return ELSA_OK;
    elsa::CombineParams cp{part_m, part_S, part_W, out, nullptr, (long long)B * H * n, n, num_splits, 1, dtype == ELSA_F16};
    return elsa::launch_combine(cp, d, static_cast<hipStream_t>(stream)) == 0 ? ELSA_OK : ELSA_ERR_HIP;
}

size_t elsa_stream_state_bytes(int B, int H, int n_q, int d) { return elsa_split_kv_workspace_bytes(B, H, n_q, d, 1); }

int elsa_attn_stream_step(const void *q, const void *k_chunk, const void *v_chunk, void *state,
                          int B, int H, int n_q, int n_chunk, int d, float scale,
                          int causal, int causal_shift, const int32_t *kv_len, int first,
                          int dtype, void *stream) {
    if (!q || !k_chunk || !v_chunk || !state) return ELSA_ERR_INVALID_ARG;
    if (!std::isfinite(scale) || n_chunk <= 0) return ELSA_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(state) & 255) return ELSA_ERR_WORKSPACE;
    const int rc = check_common(B, H, n_q, d, dtype);
    if (rc != ELSA_OK) return rc;
    float *pm, *pS, *pW;
    carve(state, B, H, n_q, d, 1, &pm, &pS, &pW);
    Extra x;
    x.nk = n_chunk;
    x.accumulate = first ? 0 : 1;
    x.has_coff = true;
    x.coff = causal_shift;
    // one chunk per call, maxima kept in log2 units so that re-merging adds no rounding of m
    return run_forward(q, k_chunk, v_chunk, nullptr, pm, pS, pW, B, H, n_q, d, scale, causal, kv_len, 1, 1, 0, dtype,
                       stream, x);
}

int elsa_attn_stream_finish(const void *state, void *out, float *lse, int B, int H, int n_q, int d, int dtype,
                            void *stream) {
    if (!state || !out) return ELSA_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(state) & 255) return ELSA_ERR_WORKSPACE;
    const int rc = check_common(B, H, n_q, d, dtype);
    if (rc != ELSA_OK) return rc;
    float *pm, *pS, *pW;
    carve(const_cast<void *>(state), B, H, n_q, d, 1, &pm, &pS, &pW);
    if (g.opt[ELSA_OPT_DRY_RUN]) return ELSA_OK;
    elsa::CombineParams cp{pm, pS, pW, out, lse, (long long)B * H * n_q, n_q, 1, 0, dtype == ELSA_F16};
    return elsa::launch_combine(cp, d, static_cast<hipStream_t>(stream)) == 0 ? ELSA_OK : ELSA_ERR_HIP;
}

int elsa_set_option(int option, int value) {
    if (option < 0 || option > 5) return ELSA_ERR_UNSUPPORTED;
    if (value < 0) return ELSA_ERR_INVALID_ARG;
    if (option == ELSA_OPT_DRY_RUN && value > 1) return ELSA_ERR_INVALID_ARG;
    if (option == ELSA_OPT_PATH && value > 3) return ELSA_ERR_INVALID_ARG;
    if (option == ELSA_OPT_XCD_MAP && value > 2) return ELSA_ERR_INVALID_ARG;
    if (option == ELSA_OPT_SNAKE && value > 1) return ELSA_ERR_INVALID_ARG;
    if (option == ELSA_OPT_SPLITS && value > kMaxSplits) return ELSA_ERR_INVALID_ARG;
    if (option == ELSA_OPT_VARIANT && value > 32) return ELSA_ERR_INVALID_ARG;
    g.opt[option] = value;
    return ELSA_OK;
}

int elsa_get_option(int option, int *value) {
    if (option < 0 || option > 5) return ELSA_ERR_UNSUPPORTED;
    if (!value) return ELSA_ERR_INVALID_ARG;
    *value = g.opt[option];
    return ELSA_OK;
}

int elsa_attn_fwd_varlen(const void *q, const void *k, const void *v, void *out,
                         const int32_t *cu_seqlens, int num_seqs, int total_tokens, int max_seqlen,
                         int H, int d, float scale, int causal, int dtype, void *stream) {
    if (!q || !k || !v || !out || !cu_seqlens) return ELSA_ERR_INVALID_ARG;
    if (!std::isfinite(scale)) return ELSA_ERR_INVALID_ARG;
    if (num_seqs <= 0 || num_seqs > kMaxSeqs || total_tokens <= 0 || max_seqlen <= 0 || max_seqlen > total_tokens)
        return ELSA_ERR_INVALID_ARG;
    const int rc = check_common(1, H, total_tokens, d, dtype);
    if (rc != ELSA_OK) return rc;
    if (((long long)total_tokens / 32 + num_seqs) * (long long)H > 0x7fffff00LL) return ELSA_ERR_INVALID_ARG;
    // tile choice as for one sequence holding every token plus half a wasted tile per sequence
    // (about the number of blocks the packed batch really yields); no key split on this path
    const long long n_eff = (long long)total_tokens + 64LL * num_seqs;
    (void)max_seqlen;
    Extra x;
    x.cu_seqlens = cu_seqlens;
    x.num_seqs = num_seqs;
    x.total_tokens = total_tokens;
    // Causal packed batches of a few runs of blocks and sequences of 512 tokens or more on average: the 64-row tile (two query x two
    // key waves) halves the longest blocks, which set the launch time (measured, 8 x U[256,1792], H = 12: 170 -> 119 us in FP32,
    // 36.9 -> 29.0 in FP16; 8 x U[512,2048], H = 8: 201 -> 138); shorter sequences, d = 128 and launches without a mask lose with it.
    if (causal && d <= 64 && (long long)total_tokens >= 512LL * num_seqs && (n_eff + 127) / 128 * H <= 6 * kNumCu) {
        const bool fp16_tiles = dtype == ELSA_F16 && scale != 0.f && (g.opt[ELSA_OPT_PATH] == 0 || g.opt[ELSA_OPT_PATH] == 3);
        x.variant = fp16_tiles ? 4 : 11;
    }
    return run_forward(q, k, v, out, nullptr, nullptr, nullptr, 1, H, (int)(n_eff > 0x7fffffff ? 0x7fffffff : n_eff), d,
                       scale, causal, nullptr, 1, 0, 0, dtype, stream, x);
}

const char *elsa_variant_name(int path, int variant) {
    return path == 1 ? elsa::fma_variant_name(variant)
         : path == 3 ? elsa::mfma16_variant_name(variant) : elsa::mfma_variant_name(variant);
}

const char *elsa_last_kernel(void) { return g.last; }

int elsa_last_splits(void) { return g.last_splits; }

const char *elsa_status_string(int code) {
    switch (code) {
        case ELSA_OK: return "ok";
        case ELSA_ERR_INVALID_ARG: return "invalid argument";
        case ELSA_ERR_UNSUPPORTED: return "unsupported head dimension, dtype or option";
        case ELSA_ERR_WORKSPACE: return "workspace too small or misaligned";
        case ELSA_ERR_HIP: return "HIP launch failure";
        default: return "unknown status";
    }
}

// Test hook (not part of the attention path): runs the device layout probe, see elsa_combine.hip.
int elsa_debug_layout_probe(float *out_5x16x64, void *stream) {
    if (!out_5x16x64) return ELSA_ERR_INVALID_ARG;
    return elsa::launch_probe(out_5x16x64, static_cast<hipStream_t>(stream)) == 0 ? ELSA_OK : ELSA_ERR_HIP;
}

// Measurement hook (not part of the attention path): runs the instruction issue-rate probe, see elsa_probe.hip.
int elsa_debug_issue_probe(float *out, int kind_a, int kind_b, int waves_per_simd, int iters, void *stream) {
    if (!out) return ELSA_ERR_INVALID_ARG;
    const int rc = elsa::launch_issue_probe(out, kind_a, kind_b, waves_per_simd, iters, static_cast<hipStream_t>(stream));
    return rc == 0 ? ELSA_OK : rc == (int)hipErrorInvalidValue ? ELSA_ERR_INVALID_ARG : ELSA_ERR_HIP;
}

}  // extern "C"
