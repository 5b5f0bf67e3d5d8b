// ELSA forward with value rows of their own width (d_v != d), FP16 I/O on the FP16 matrix cores:
// the tile configurations of the (d, d_v) pairs served and their launchers.
#include "elsa_fwd_mfma16_kernel.hpp"

namespace elsa {

template <int D, int DV>
static int launch_dv16(const FwdParams &p, int variant, hipStream_t s) {
    if (variant == 3) {
        if constexpr (D <= 64 && DV <= 64) return launch_one16<D, 1, 1, 4, 32, 2, DV>(p, s);
        else return launch_one16<D, 1, 2, 2, 32, 2, DV>(p, s);
    }
    if (variant == 6) {
        // eight query waves (256 rows) on shared tiles, one block per CU: the staging of the wide rows is paid once for
        // twice the query rows.  128-key tiles where a 32-column operand would not give every thread a whole chunk.
        if constexpr (D >= 128 || DV >= 128) return launch_one16<D, 1, 8, 1, (D == 32 || DV == 32) ? 128 : 64, 2, DV>(p, s);
        else return (int)hipErrorInvalidValue;
    }
    // 64-key LDS tiles; 32 at d = 192, so that two blocks of a CU fit its LDS
    constexpr int KS = D == 192 ? 32 : 64;
    return launch_one16<D, 1, 4, 1, KS, 2, DV>(p, s);
}

int launch_fwd_dv16(const FwdParams &p, int d, int dv, int variant, hipStream_t s, const char **name) {
    if (name) *name = variant == 3 ? "mfma16_dv_xwave" : variant == 6 ? "mfma16_dv_q256_w8" : "mfma16_dv_q128";
    if (variant != 1 && variant != 3 && variant != 6) return (int)hipErrorInvalidValue;
#define ELSA_DV_CASE(DD, VV) \
    if (d == DD && dv == VV) return launch_dv16<DD, VV>(p, variant, s);
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
