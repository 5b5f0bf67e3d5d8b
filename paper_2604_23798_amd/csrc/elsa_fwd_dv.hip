// ELSA forward with value rows of their own width (d_v != d), FP32 matrix cores: the tile
// configurations of the (d, d_v) pairs served and their launchers.  The kernel is the one of the
// d_v = d path: d sets the contraction of the scores, d_v the rows of W^T.
#include "elsa_fwd_mfma_kernel.hpp"

namespace elsa {

// tile ids: 1 = 128 query rows (four query waves, 32-key LDS tiles)
//           3 = the waves of a block split the key range (32 query rows when d, d_v <= 64, else 64)
//           6 = FP16 tiles with d or d_v >= 128 only: 256 query rows, eight query waves on shared K/V tiles
int dv_variant_tq(int fp16_tiles, int variant, int d, int dv) {
    if (variant == 1) return 128;
    if (variant == 6) return (fp16_tiles && (d >= 128 || dv >= 128)) ? 256 : 0;
    if (variant != 3) return 0;
    if (!fp16_tiles && d == 192) return 0;       // two FP32 tiles of 64 keys x (192 + 128) columns exceed the LDS
    return (d <= 64 && dv <= 64) ? 32 : 64;
}

template <int D, int DV, typename T>
static int launch_dv32(const FwdParams &p, int variant, hipStream_t s) {
    constexpr bool small = D <= 64 && DV <= 64;
    if (variant == 3) {
        if constexpr (D == 192) return (int)hipErrorInvalidValue;
        else if constexpr (small) return launch_one<D, T, 1, 1, 4, 32, 2, 2, 1, DV, 1>(p, s);
        else return launch_one<D, T, 1, 2, 2, 32, 1, 2, 1, DV, 1>(p, s);   // its tiles leave room for one block per CU: no register cap
    }
    // waves per SIMD the registers allow: three for the narrow pairs, one at d = 192
    constexpr int WPE = D == 192 ? 1 : small ? 3 : 2;
    // (last argument: the lagging reference of the d_v = d tiles; every pair has the sixteen registers it needs)
    return launch_one<D, T, 1, 4, 1, 32, WPE, 2, 1, DV, 1>(p, s);
}

int launch_fwd_dv32(const FwdParams &p, int d, int dv, int f16, int variant, hipStream_t s, const char **name) {
    if (name) *name = variant == 3 ? "mfma_dv_xwave" : "mfma_dv_q128";
    if (variant != 1 && variant != 3) return (int)hipErrorInvalidValue;
#define ELSA_DV_CASE(DD, VV) \
    if (d == DD && dv == VV) return f16 ? launch_dv32<DD, VV, _Float16>(p, variant, s) : launch_dv32<DD, VV, float>(p, variant, s);
    ELSA_DV_CASE(32, 64)
    ELSA_DV_CASE(32, 128)
    ELSA_DV_CASE(64, 32)
    ELSA_DV_CASE(64, 128)
    ELSA_DV_CASE(128, 32)
    ELSA_DV_CASE(128, 64)
    ELSA_DV_CASE(192, 128)
#undef ELSA_DV_CASE
    return (int)hipErrorInvalidValue;
}

}  // namespace elsa
