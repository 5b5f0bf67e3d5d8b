// The host planner of libelsa (csrc/elsa_plan.cpp: fixed stack arrays, a hand-rolled heap, per-shape
// tables) under AddressSanitizer and UBSan: this driver is compiled together with that file and sweeps
// it over the documented shapes plus a seeded random grid (B*H 1 .. 4096, n 1 .. 2^20, every head
// dimension, both masks, both tile families, with and without a workspace).  Every answer must be a
// tile id of its family and a chunk count the keys and the workspace allow; the sanitizers stop the
// run on any out-of-bounds index or overflow on the way.  Exit status 0 = all held.
#include <cstdint>
#include <cstdio>

#include "elsa_plan.hpp"

using namespace elsa::plan;

static int fails = 0;
#define CHECK(cond)                                                          \
    do {                                                                     \
        if (!(cond)) {                                                       \
            std::printf("FAILED %s:%d %s\n", __FILE__, __LINE__, #cond);     \
            ++fails;                                                         \
        }                                                                    \
    } while (0)

static uint64_t state = 0x9E3779B97F4A7C15ULL;
static uint64_t next() {
    state ^= state << 13; state ^= state >> 7; state ^= state << 17;
    return state;
}
static int log_uniform(int lo_log2, int hi_log2) {          // 2^lo .. 2^hi, any value in between
    const int e = lo_log2 + (int)(next() % (uint64_t)(hi_log2 - lo_log2 + 1));
    const uint64_t base = 1ULL << e, top = 1ULL << hi_log2;
    const uint64_t v = base + next() % base;
    return (int)(v > top ? top : v);
}

static void one(bool fp16, long long BH, int n, int nk, int d, int causal, int max_c) {
    const TileChoice tc = choose_tiles(fp16, BH, n, nk, d, causal, max_c);
    CHECK(tc.variant >= 1 && tc.variant <= (fp16 ? 4 : 13));
    CHECK(tc.splits >= 1 && tc.splits <= max_c);
    CHECK(tc.splits == 1 || nk / tc.splits >= 256);
    const TileChoice again = choose_tiles(fp16, BH, n, nk, d, causal, max_c);      // remembered answer
    CHECK(again.variant == tc.variant && again.splits == tc.splits);
}

static void one_dv(bool fp16, long long BH, int n, int nk, int d, int dv, int causal, int max_c) {
    const TileChoice tc = choose_tiles_dv(fp16, BH, n, nk, d, dv, causal, max_c);
    CHECK(tc.variant == 1 || tc.variant == 3);
    CHECK(tc.splits >= 1 && tc.splits <= max_c);
}

int main() {
    // workspace sizes
    CHECK(workspace_bytes(1, 12, 197, 64, 4) == 2 * ((size_t)(12 * 4 * 197 * 4 + 255) / 256 * 256) + (size_t)12 * 4 * 197 * 64 * 4);
    CHECK(workspace_bytes(1, 12, 197, 48, 4) == 0 && workspace_bytes(0, 1, 1, 64, 1) == 0 && workspace_bytes(1, 1, 1, 64, 0) == 0);
    CHECK(workspace_bytes(4096, 64, 1 << 20, 256, 65535) > 0);                     // no overflow trap on the way

    // documented shapes
    const int dims[5] = {32, 64, 96, 128, 256};
    const int ns[9] = {1, 9, 197, 512, 1024, 1536, 3072, 8192, 16384};
    const long long bhs[7] = {1, 8, 12, 16, 40, 192, 768};
    for (int fp16 = 0; fp16 < 2; ++fp16)
        for (int d : dims)
            for (int n : ns)
                for (long long BH : bhs)
                    for (int causal = 0; causal < 2; ++causal)
                        for (int max_c = 1; max_c <= 4; max_c += 3) one(fp16 != 0, BH, n, n, d, causal, max_c);

    // seeded random shapes, square and rectangular
    for (int it = 0; it < 4000; ++it) {
        const bool fp16 = next() & 1;
        const int d = dims[next() % 5];
        const long long BH = log_uniform(0, 12);
        const int n = log_uniform(0, 20);
        const int nk = (next() & 3) ? n : log_uniform(0, 20);
        const int causal = (int)(next() & 1);
        const int max_c = 1 + (int)(next() % 8);
        // the play-through walks every block of the launch: keep the sweep to launches it is meant for
        // (the library calls it for at most 12 x 256 blocks of 128 rows) plus a margin
        if (BH * ((n + 31) / 32) > 400000) continue;
        one(fp16, BH, n, nk, d, causal, max_c);
        // the wide FP16 tile is never chosen below d = 96 nor for fewer blocks than half the CUs
        const bool wide = wide_fp16_tile_pays(BH, n, d, causal);
        CHECK(!wide || (d >= 96 && BH * ((n + 255) / 256) >= kCus / 2));          // (d = 256 from half the CUs, else from 5/8)
        static const int pairs[7][2] = {{32, 64}, {64, 32}, {64, 128}, {128, 64}, {32, 128}, {128, 32}, {192, 128}};
        const int *pr = pairs[next() % 7];
        one_dv(fp16, BH, n, nk, pr[0], pr[1], causal, max_c);
    }

    CHECK(wide_fp16_tile_pays(40, 32768, 128, 1) && wide_fp16_tile_pays(16, 8192, 128, 0) && !wide_fp16_tile_pays(40, 2048, 128, 0));
    CHECK(!wide_fp16_tile_pays(16, 16384, 64, 0) && !wide_fp16_tile_pays(0, 1024, 128, 0) && !wide_fp16_tile_pays(4096, 1 << 20, 128, 1) == false);

    // chunk counts: never more than the keys or the workspace allow, never below one
    for (int it = 0; it < 20000; ++it) {
        const int B = log_uniform(0, 6), H = log_uniform(0, 6);
        const int n = log_uniform(0, 20), nk = (next() & 1) ? n : log_uniform(0, 20);
        const int d = dims[next() % 5];
        const size_t ws = (size_t)(next() % 5 == 0 ? 0 : (next() % (1ULL << 32)));
        const int requested = (next() & 3) ? 0 : (int)(next() % 70000);
        const int C = auto_splits(requested, B, H, n, nk, d, next() & 1, ws);
        CHECK(C >= 1 && C <= kMaxSplits && C <= (nk > 1 ? nk : 1));
        CHECK(C == 1 || workspace_bytes(B, H, n, d, C) <= ws);
        if (requested > 0) CHECK(C <= requested);
    }
    std::printf("%s\n", fails ? "planner under sanitizers: FAILED" : "planner under sanitizers: ok");
    return fails ? 1 : 0;
}
