// Launch planning on the host: tile shape and key chunks of small dense problems.  Plain C++, no HIP.
#include "elsa_plan.hpp"

#include <algorithm>
#include <functional>

namespace elsa {
namespace plan {

namespace {

constexpr int kNumCu = kCus;

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
bool head_dim_ok(int d) { return d == 32 || d == 64 || d == 96 || d == 128 || d == 256; }

// Tile shape and number of key chunks for small dense problems, where the choice decides how evenly
// the blocks fill the 256 CUs.  The launch is played through on the host: a block's work is its
// 32-key steps per wave (for the block's place in the launch order, masks included); the first
// `resident` x 256 blocks are placed round-robin as the hardware does, later ones go to the CU that
// frees up first; blocks that share a CU add up, because the matrix core and the vector ALU of a
// SIMD take turns.  Launch time = steps of the busiest CU x step time + prologue (+ state traffic
// and the combine launch when the keys are cut).  Step times are measured (us per step at d = 64;
// t2 when co-resident blocks overlap, t1 when a block is alone or its neighbours differ in length):
//   FP32  128 rows 2.25 / 2.0   64 rows x 2 key waves 2.4 / 2.15   32 rows x 4 key waves 2.6
//   FP16  128 rows 0.54 / 0.36  256 rows 0.88 / 0.66  64 rows x 2 key waves 0.60 / 0.40  32 rows x 4: 0.58
// Predictions are within about 10 % of the measured launch times on B*H = 8 .. 192, n = 197 .. 4096.
struct TileShape { int variant, rows, key_waves, resident; double t1, t2; };

// The play-through itself, for a table of tile shapes.  `dw` is the width of a chunk state's W (d, or d_v when the
// values have a width of their own); `no_cut` marks shapes that are never cut (bit i = shape i).
TileChoice play_through(const TileShape *shapes, int nshapes, double dscale, unsigned no_cut, bool fp16_tiles, long long BH, int n,
                        int nk, int dw, int causal, int max_splits) {
    const double prologue = 5.0;
    const int coff = nk - n;
    TileChoice best{shapes[0].variant, 1};
    double best_t = 1e30;
    double cu[kNumCu];                       // work placed on each CU (steps)
    double free_at[kNumCu];                  // min-heap: when a CU takes its next block (no host allocation)
    for (int si = 0; si < nshapes; ++si) {
        const TileShape &sh = shapes[si];
        // under a causal mask the 256-row tile's diagonal tiles waste twice as much: measured best only on long sequences
        // with at least 1024 such blocks (n >= 16384: 1.04-1.07 of the 128-row tile's speed; shorter or fewer: 0.83-0.98)
        if (fp16_tiles && sh.rows == 256 && causal && !(n >= 16384 && BH * ((n + 255) / 256) >= 4 * kNumCu)) continue;
        if (!fp16_tiles && sh.variant == 13 && nk < 1024) continue;   // the single-buffered tile pays from about sixteen 64-key tiles per block up
        const int q_tiles = (n + sh.rows - 1) / sh.rows;
        for (int C = 1; C <= max_splits; ++C) {
            if (C > 1 && (((no_cut >> si) & 1u) || nk / C < 256)) break;
            // under a causal mask key chunks only pay while the 128-row blocks do not fill the CUs twice: measured
            // 20-45 % slower than one pass from two runs of blocks up (H = 8, n = 16384: 2.6 against 2.1 ms)
            if (C > 1 && causal && sh.resident >= 2 && BH * ((n + 127) / 128) >= 2 * kNumCu) break;
            const int chunk = (nk + C - 1) / C;
            const long long blocks = BH * q_tiles * C;
            if (blocks > 64 * kNumCu) continue;          // not a small problem in this shape
            auto steps_of = [&](int qt, int c) {
                int hi = nk < (c + 1) * chunk ? nk : (c + 1) * chunk;
                if (causal) { const int lim = (qt + 1) * sh.rows + coff; if (lim < hi) hi = lim; }
                const int vis = hi - c * chunk;
                return vis > 0 ? (vis + 32 * sh.key_waves - 1) / (32 * sh.key_waves) : 0;
            };
            // per-block cost in steps: a tile that owns its CU pays its prologue itself; co-resident blocks hide most of each
            // other's, what is left (Q fragments, first tile, epilogue; the merge of the key waves' states) was measured on
            // batches of short sequences: about 0.9 us per block at d = 64, 1.3 us when the waves split the keys, growing with d
            const double own = sh.resident == 1 ? prologue / (sh.t1 * dscale)
                                                : (sh.key_waves > 1 ? 1.3 : 0.9) * (0.5 + dw / 128.0) / (sh.t2 * dscale);
            std::fill(cu, cu + kNumCu, 0.0);
            int heap_n = 0;
            const long long placed = (long long)sh.resident * kNumCu;
            for (long long i = 0; i < blocks; ++i) {
                long long w = i;                          // launch order: see decode_work (head index fastest)
                if (causal) {
                    if (sh.resident == 3 && blocks > 3 * kNumCu && blocks <= 4 * kNumCu) { const long long half = blocks / 2; if (w >= half) w = half + (blocks - 1 - w); }
                    else if (w >= kNumCu && w < 2 * kNumCu) { const long long last = blocks < 2 * kNumCu ? blocks : 2 * kNumCu; w = kNumCu + (last - 1 - w); }
                }
                const long long t = w / BH;
                int qt = (int)(t % q_tiles);
                const int c = (int)(t / q_tiles);
                if (causal) qt = q_tiles - 1 - qt;
                const double cost = steps_of(qt, c) + own;
                if (i < placed) {
                    cu[i % kNumCu] += cost;
                    if (i + kNumCu >= placed || i + kNumCu >= blocks) {   // the CU's last static block
                        free_at[heap_n++] = cu[i % kNumCu];
                        std::push_heap(free_at, free_at + heap_n, std::greater<double>());
                    }
                } else {
                    std::pop_heap(free_at, free_at + heap_n, std::greater<double>());   // earliest CU to the back
                    free_at[heap_n - 1] += cost;
                    std::push_heap(free_at, free_at + heap_n, std::greater<double>());
                }
            }
            double busiest = 0.0;
            if (blocks <= placed) busiest = *std::max_element(cu, cu + kNumCu);
            else busiest = *std::max_element(free_at, free_at + heap_n);
            const long long rounds = (blocks + kNumCu - 1) / kNumCu;
            const bool overlap = sh.resident >= 2 && (causal ? rounds > sh.resident : rounds >= 2);
            const double step = (overlap ? sh.t2 : sh.t1) * dscale;
            // second launch + the chunk states written and read back ((d + 2) floats per row and chunk, ~4 TB/s)
            const double combine = C > 1 ? 5.0 + 2.0 * (double)(rounds - 1) + (double)BH * n * C * (dw + 2) * 8.0 / 4.0e6 : 0.0;
            const double t = (sh.resident == 1 ? 0.0 : prologue) + busiest * step + combine;
            if (t < best_t) { best_t = t; best = TileChoice{sh.variant, C}; }
        }
    }
    return best;
}

}  // namespace

TileChoice choose_tiles(bool fp16_tiles, long long BH, int n, int nk, int d, int causal, int max_splits) {
    // the last question is usually asked again (a layer stack, a benchmark loop): remember its answer
    struct Memo { bool f16; long long BH; int n, nk, d, causal, max_splits; TileChoice choice; };
    static thread_local Memo memo{false, -1, 0, 0, 0, 0, 0, {0, 0}};   // per host thread: no lock needed
    if (memo.f16 == fp16_tiles && memo.BH == BH && memo.n == n && memo.nk == nk && memo.d == d && memo.causal == causal &&
        memo.max_splits == max_splits)
        return memo.choice;
    static const TileShape f32_narrow[3] = {{7, 128, 1, 3, 2.25, 2.0}, {11, 64, 2, 2, 2.4, 2.15}, {3, 32, 4, 1, 2.6, 2.6}};
    // d = 128: the 128-row tile holds two blocks per CU, the 64-row tile (its LDS tiles fill a CU) one
    // (one wave per SIMD hides no latency: 5.3 us per step at d = 128, 2.8 at the d = 64 scale)
    // the same 64-row tile single-buffered [13]: half the LDS, two blocks per CU; slower alone (2.9), faster in pairs (2.5); never cut (measured 10-20 % behind the cut 128-row tile)
    static const TileShape f32_wide[3] = {{1, 128, 1, 2, 2.4, 2.15}, {11, 64, 2, 1, 2.8, 2.8}, {13, 64, 2, 2, 2.9, 2.5}};
    static const TileShape f16_narrow[4] = {{1, 128, 1, 2, 0.54, 0.36}, {2, 256, 1, 2, 0.88, 0.66}, {4, 64, 2, 2, 0.60, 0.40},
                                            {3, 32, 4, 2, 0.58, 0.58}};
    // FP16 tiles at d = 128 (us per step as measured there, not scaled): 128 rows 0.78 / 0.64; 64 rows x 2 key waves 1.0 / 0.75
    static const TileShape f16_wide[2] = {{1, 128, 1, 2, 0.78, 0.64}, {4, 64, 2, 2, 1.0, 0.75}};
    // d = 96: the FP32 128-row tile behaves as at d = 128; its 64-row tile (two query x two key waves) owns the CU (100 KB of LDS);
    // d = 256: one FP32 shape, one wave per SIMD.  FP16 at d = 96, unscaled: 128 rows 0.71 / 0.53, 64 rows x 2 key waves 0.80 / 0.60.
    static const TileShape f32_d96[2] = {{1, 128, 1, 2, 2.4, 2.15}, {3, 64, 2, 1, 2.66, 2.66}};
    static const TileShape f32_d256[1] = {{1, 128, 1, 1, 2.75, 2.62}};
    static const TileShape f16_d96[2] = {{1, 128, 1, 2, 0.71, 0.53}, {4, 64, 2, 2, 0.80, 0.60}};
    // FP16 at d = 256: the 128-row tile (register-capped, two blocks per CU) is slow alone: 2.8 / 1.41; 64 rows x 2 key waves own the CU: 2.3 / 2.0
    static const TileShape f16_d256[2] = {{1, 128, 1, 2, 2.8, 1.41}, {4, 64, 2, 1, 2.3, 2.0}};
    const TileShape *shapes = fp16_tiles ? (d == 128 ? f16_wide : d == 96 ? f16_d96 : d == 256 ? f16_d256 : f16_narrow)
                                         : d == 128 ? f32_wide : d == 96 ? f32_d96 : d == 256 ? f32_d256 : f32_narrow;
    const int nshapes = fp16_tiles ? (d >= 96 ? 2 : 4) : d == 96 ? 2 : d == 256 ? 1 : 3;
    const double dscale = (fp16_tiles && d >= 96) ? 1.0 : 0.12 + 0.88 * d / 64.0;        // the MFMA part of a step grows with d
    // never cut: the FP32 32-row tile (its four waves split the keys already) and the single-buffered 64-row tile
    unsigned no_cut = 0;
    for (int si = 0; si < nshapes; ++si)
        if (!fp16_tiles && ((shapes[si].variant == 3 && shapes[si].key_waves == 4) || shapes[si].variant == 13)) no_cut |= 1u << si;
    const TileChoice best = play_through(shapes, nshapes, dscale, no_cut, fp16_tiles, BH, n, nk, d, causal, max_splits);
    memo = Memo{fp16_tiles, BH, n, nk, d, causal, max_splits, best};
    return best;
}

// The same choice when the values have a width of their own: tiles 1 (128 rows) and 3 (the waves split the keys: 32 rows x four
// key waves when d, d_v <= 64, else 64 rows x two).  A step costs what the d_v = d tiles cost at the mean width (d + d_v) / 2
// (scores contract over d, W^T has d_v rows); FP16 step times interpolate the measured ones of d = 64, 96, 128.
TileChoice choose_tiles_dv(bool fp16_tiles, long long BH, int n, int nk, int d, int dv, int causal, int max_splits) {
    struct Memo { bool f16; long long BH; int n, nk, d, dv, causal, max_splits; TileChoice choice; };
    static thread_local Memo memo{false, -1, 0, 0, 0, 0, 0, 0, {0, 0}};
    if (memo.f16 == fp16_tiles && memo.BH == BH && memo.n == n && memo.nk == nk && memo.d == d && memo.dv == dv &&
        memo.causal == causal && memo.max_splits == max_splits)
        return memo.choice;
    const double x = 0.5 * (d + dv) / 64.0;
    const bool narrow = d <= 64 && dv <= 64;
    TileShape shapes[2];
    int nshapes = 2;
    double dscale = 1.0;
    if (fp16_tiles) {
        shapes[0] = TileShape{1, 128, 1, 2, 0.30 + 0.24 * x, 0.08 + 0.28 * x};
        if (narrow) shapes[1] = TileShape{3, 32, 4, 2, 0.1 + 0.48 * x, 0.1 + 0.48 * x};
        else if (d == 192) shapes[1] = TileShape{3, 64, 2, 2, 1.5, 1.26};     // measured: slower than the interpolation at this width
        else shapes[1] = TileShape{3, 64, 2, 2, 0.20 + 0.40 * x, 0.05 + 0.35 * x};
    } else {
        dscale = 0.12 + 0.88 * x;
        if (d == 192) { shapes[0] = TileShape{1, 128, 1, 1, 2.75, 2.62}; nshapes = 1; }
        else if (narrow) { shapes[0] = TileShape{1, 128, 1, 3, 2.25, 2.0}; shapes[1] = TileShape{3, 32, 4, 1, 2.6, 2.6}; }
        else { shapes[0] = TileShape{1, 128, 1, 2, 2.4, 2.15}; shapes[1] = TileShape{3, 64, 2, 1, 2.8, 2.8}; }
    }
    const unsigned no_cut = (!fp16_tiles && narrow) ? 2u : 0u;
    const TileChoice best = play_through(shapes, nshapes, dscale, no_cut, fp16_tiles, BH, n, nk, dv, causal, max_splits);
    memo = Memo{fp16_tiles, BH, n, nk, d, dv, causal, max_splits, best};
    return best;
}

// The 256-row FP16 tile of eight query waves owns a CU (two waves per SIMD, like two 128-row blocks) and stages every K/V
// tile once for 256 rows instead of twice.  Staging is 19 % of the 128-row tile's time at d = 128 and more at d = 256, so
// the wide tile wins wherever its coarser blocks still fill the CUs evenly.  Measured on B = 1, H = 8 / 16 / 40,
// n = 1024 ... 16384 (ratio 128-row / 256-row time; b = number of 256-row blocks):
//   d = 128, no mask: b = 128 0.86, 160 1.18 (against the 64-row tile the planner picks there), 256 1.06-1.14, 512 1.12, 1024 1.09, 1280 1.10, 2560 1.05; but 320 0.91, 640 0.99 (2.5 rounds of
//            256 blocks cost 3); d = 96 the same picture (256: 1.02-1.08, 512: 1.12-1.13, 320: 0.90, 640: 0.95)
//   d = 128 / 96, causal: 1024 1.05-1.08, 1280 1.02-1.04, 2560 1.05, 32K x 40 heads 1.07; 512 0.90-0.95
//   d = 256: no mask 1.03-1.05 at b = 128, 1.23-1.37 from 160 up; causal 1.08-1.32 from b = 256 up, 0.74-0.87 below
bool wide_fp16_tile_pays(long long BH, int n, int d, int causal) {
    if (d < 96 || BH <= 0 || n <= 0) return false;
    const long long b = BH * ((n + 255) / 256);
    if (d == 256) return causal ? b >= kCus : b >= kCus / 2;
    if (causal) return b >= 4 * kCus;
    if (b < kCus) return 8 * b >= 5 * kCus;          // one partial round: from 160 blocks up (1.13-1.18 at 160, 0.86 at 128)
    const long long rounds = (b + kCus - 1) / kCus;
    return 100 * b >= 88 * rounds * kCus;            // the last round of blocks is at least ~90 % full on average
}

size_t workspace_bytes(int B, int H, int n, int d, int num_splits) {
    if (B <= 0 || H <= 0 || n <= 0 || !head_dim_ok(d) || num_splits < 1) return 0;
    const size_t rows = (size_t)B * H * num_splits * n;
    return 2 * align256(rows * 4) + align256(rows * d * 4);
}

// Number of key chunks for elsa_attn_fwd when a workspace is lent: enough 128-row blocks for
// one per CU, chunks no shorter than 256 keys, at most 8 (64 when decoding), and only if the
// workspace holds them.
int auto_splits(int requested, int B, int H, int n, int nk, int d, bool fp16_tiles, size_t ws_bytes) {
    int C = requested;
    if (C <= 0) {
        const long long blocks = (long long)B * H * ((n + 127) / 128);
        C = 1;
        // few queries against many keys (decoding): the key range is the only parallelism; about
        // five blocks per CU measured best there.  Otherwise one block per CU: every further cut
        // adds prologue, state traffic and combine work without adding matrix-core throughput
        // (measured at n = 1024, H = 16: 2 chunks 47.5 us, 4 chunks 51 us, none 77 us).
        const bool few_q = (long long)n * 8 <= nk;
        const int want = few_q ? 5 * kNumCu : kNumCu;
        // The FP16 tiles are so much faster per key that, outside decoding, a second launch costs more
        // than idle CUs do (n = 1024, H = 16: 13.4 us in one pass of the key-splitting tile, 20 us cut
        // in two; n = 2048: 39.6 against 41.6 us).
        if (blocks <= want && (few_q || !fp16_tiles)) {
            C = (int)((want + blocks - 1) / blocks);
            if (C < 2) C = 2;                    // exactly one block per CU still gains from two chunks
            const int cap = nk / 256 > 1 ? nk / 256 : 1;
            if (C > cap) C = cap;
            const int most = few_q ? 64 : 8;
            if (C > most) C = most;
        }
    }
    if (C > nk) C = nk;
    if (C > kMaxSplits) C = kMaxSplits;
    while (C > 1 && workspace_bytes(B, H, n, d, C) > ws_bytes) --C;
    return C < 1 ? 1 : C;
}

}  // namespace plan
}  // namespace elsa
