// ELSA forward, FP32 MFMA path (gfx950): tile configurations and their launchers for d_v = d.
#include "elsa_fwd_mfma_kernel.hpp"

namespace elsa {

// ---- variants -------------------------------------------------------------------------------
// id: 1 q128: 4 query waves, 64-key tiles            2 q256: 4 query waves x 2 query groups
//     3 xwave: the waves split the key range          4 q256w8: 8 query waves, 32-key tiles (4 per SIMD)
//     5 q128 with 1 score chain                       6 q128 with 4 score chains
//     7 q128k32: 32-key tiles, 3 waves per SIMD       8 q128 with plain global loads (no descriptors)
// All but 8 fetch tiles through buffer descriptors; all but 5/6 use 2 score chains.
//     9/10 small: one wave per 64 / 32 query rows, operands straight from memory (elsa_fwd_small.hip)
//     11 q64xw2: 64 query rows, two query waves x two key waves (the key-splitting shape of d >= 96)
//     12 xwave32: d = 128 only: 32 query rows, four key waves on one 128-key LDS tile (single buffer)
//     13 q64xw2sb: d = 128 only: shape 11 with a single LDS buffer (67 KB), so that two blocks share a CU

static const char *kNames[kMfmaVariants] = {"mfma_q128_w4",   "mfma_q256_w4",   "mfma_xwave",    "mfma_q256_w8",
                                            "mfma_q128_acc1", "mfma_q128_acc4", "mfma_q128_k32", "mfma_q128_gld",
                                            "mfma_small_q64", "mfma_small_q32", "mfma_q64_xw2", "mfma_xwave32",
                                            "mfma_q64_xw2_sb"};

int mfma_variant_tq(int variant, int d) {
    switch (variant) {
        case 1: case 5: case 6: case 7: case 8: return 128;
        case 2: return d <= 64 ? 256 : 128;
        case 4: return d <= 64 ? 256 : 128;
        case 3: return d == 256 ? 128 : d <= 64 ? 32 : 64;   // d = 96, 128: two query waves x two key waves
        case 9: return 64;                      // one wave per 64 (32) query rows, no LDS
        case 10: return 32;
        case 11: return d == 256 ? 128 : 64;
        case 12: return d == 128 ? 32 : 0;
        case 13: return d == 128 ? 64 : 0;
        default: return 0;
    }
}
const char *mfma_variant_name(int variant) {
    return (variant >= 1 && variant <= kMfmaVariants) ? kNames[variant - 1] : nullptr;
}

template <int D, typename T>
static int launch_variant(const FwdParams &p, int variant, hipStream_t s) {
    // The last template argument (1) turns on the lagging reference where the sixteen extra registers per query group
    // neither spill nor cost a resident block; the 256-row tiles, the eight-wave tile, the four-chain and the
    // single-buffered tile at d = 128 and every tile at d = 256 stay on the exact maximum per step.
    // d = 96 and d = 256: one tile shape (128 rows, 32-key tiles; two waves per SIMD at d = 96, one at
    // d = 256 where the state and the query fragment fill the register file) and, for d = 96, the
    // key-splitting shape
    if constexpr (D == 96) {
        if (variant == 3 || variant == 11) return launch_one<D, T, 1, 2, 2, 32, 2, 2, 1, D, 1>(p, s);
        return launch_one<D, T, 1, 4, 1, 32, 2, 2, 1, D, 1>(p, s);
    } else if constexpr (D == 256) {
        return launch_one<D, T, 1, 4, 1, 32, 1, 1, 1>(p, s);
    } else {
    // keys per LDS buffer: 64 for d <= 64, 32 for d = 128 (same bytes)
    constexpr int KS = D == 128 ? 32 : 64;
    switch (variant) {
        case 1: return launch_one<D, T, 1, 4, 1, KS, 2, 2, 1, D, 1>(p, s);
        case 2:
            if constexpr (D == 128) return launch_one<D, T, 1, 4, 1, KS, 2, 2, 1, D, 1>(p, s);   // no room for two query groups
            else return launch_one<D, T, 2, 4, 1, KS, 2, 2, 1>(p, s);
        case 3:
            // d = 128: two 64-key tiles of K and V fill the LDS of a CU, so one block (one wave per SIMD)
            // is resident anyway: no register cap (the cap of two waves per SIMD spilled 20 registers)
            if constexpr (D == 128) return launch_one<D, T, 1, 2, 2, 32, 1, 2, 1, D, 1>(p, s);
            else return launch_one<D, T, 1, 1, 4, 32, 2, 2, 1, D, 1>(p, s);
        case 4:
            // d = 64: 8 waves on 32-key tiles, 4 per SIMD in 128 registers.  d = 128 has no such
            // configuration (the state alone needs more registers): same as id 5.
            if constexpr (D == 64) return launch_one<D, T, 1, 8, 1, 32, 4, 2, 1>(p, s);
            else if constexpr (D == 32) return launch_one<D, T, 1, 8, 1, 64, 4, 2, 1>(p, s);
            else return launch_one<D, T, 1, 4, 1, KS, 2, 1, 1, D, 1>(p, s);
        case 5: return launch_one<D, T, 1, 4, 1, KS, 2, 1, 1, D, 1>(p, s);
        case 6: return launch_one<D, T, 1, 4, 1, KS, 2, 4, 1>(p, s);
        case 7:
            if constexpr (D == 128) return launch_one<D, T, 1, 4, 1, KS, 2, 2, 1, D, 1>(p, s);
            else return launch_one<D, T, 1, 4, 1, 32, 3, 2, 1, D, 1>(p, s);
        case 8:
            if constexpr (D == 128) return launch_one<D, T, 1, 4, 1, KS, 2, 2, 0>(p, s);     // (would spill)
            else return launch_one<D, T, 1, 4, 1, KS, 2, 2, 0, D, 1>(p, s);
        case 11:
            if constexpr (D == 128) return launch_one<D, T, 1, 2, 2, 32, 1, 2, 1, D, 1>(p, s);
            else return launch_one<D, T, 1, 2, 2, 32, 2, 2, 1, D, 1>(p, s);
        case 12:
            if constexpr (D == 128) return launch_one<D, T, 1, 1, 4, 32, 1, 2, 2, D, 1>(p, s);
            else return (int)hipErrorInvalidValue;
        case 13:
            if constexpr (D == 128) return launch_one<D, T, 1, 2, 2, 32, 2, 2, 2>(p, s);
            else return (int)hipErrorInvalidValue;
        default: return (int)hipErrorInvalidValue;
    }
    }
}

int launch_fwd_mfma(const FwdParams &p, int d, int f16, int variant, hipStream_t s, const char **name) {
    if (name) *name = mfma_variant_name(variant);
    if (variant == 9 || variant == 10) return launch_fwd_mfma_small(p, d, f16, variant == 9 ? 2 : 1, s);
    if (d == 32) return f16 ? launch_variant<32, _Float16>(p, variant, s) : launch_variant<32, float>(p, variant, s);
    if (d == 64) return f16 ? launch_variant<64, _Float16>(p, variant, s) : launch_variant<64, float>(p, variant, s);
    if (d == 128) return f16 ? launch_variant<128, _Float16>(p, variant, s) : launch_variant<128, float>(p, variant, s);
    if (d == 96) return f16 ? launch_variant<96, _Float16>(p, variant, s) : launch_variant<96, float>(p, variant, s);
    if (d == 256) return f16 ? launch_variant<256, _Float16>(p, variant, s) : launch_variant<256, float>(p, variant, s);
    return (int)hipErrorInvalidValue;
}

}  // namespace elsa
