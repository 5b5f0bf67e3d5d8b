// ELSA forward, FP16-I/O path on the FP16 matrix cores (gfx950): tile configurations and their
// launchers for d_v = d.
#include "elsa_fwd_mfma16_kernel.hpp"

namespace elsa {

// ---- variants: 1 q128 (4 query waves)   2 q256 (4 waves x 2 query groups)   3 waves split the keys
//                4 q64xw2 (two query waves x two key waves; the key-splitting shape of d >= 96)
//                5 q256 as first built: 64-key tiles, one loop body per step, no early K request (comparison; d <= 64 only)
//                6 q256w8 (d >= 96 only): eight query waves of one group each share the K/V tiles of 256 query rows, one
//                  block per CU: half the tile staging per query row of the 128-row tile

static const char *kNames16[kMfma16Variants] = {"mfma16_q128_w4", "mfma16_q256_w4", "mfma16_xwave", "mfma16_q64_xw2", "mfma16_q256_plain", "mfma16_q256_w8"};

int mfma16_variant_tq(int variant, int d) {
    switch (variant) {
        case 1: return 128;
        case 2: return d <= 64 ? 256 : 128;
        case 3: return d <= 64 ? 32 : 64;       // d >= 96: two query waves x two key waves
        case 4: return 64;
        case 5: return d <= 64 ? 256 : 0;
        case 6: return d >= 96 ? 256 : 0;
        default: return 0;
    }
}
const char *mfma16_variant_name(int variant) {
    return (variant >= 1 && variant <= kMfma16Variants) ? kNames16[variant - 1] : nullptr;
}

template <int D>
static int launch_variant16(const FwdParams &p, int variant, hipStream_t s) {
    // d = 96, 256: one query group per wave; 32-key tiles at d = 256 keep two blocks per CU in LDS
    if constexpr (D == 96) {
        if (variant == 6) return launch_one16<D, 1, 8, 1, 128, 2>(p, s);
        if (variant == 3 || variant == 4) return launch_one16<D, 1, 2, 2, 32, 2>(p, s);
        return launch_one16<D, 1, 4, 1, 64, 2>(p, s);
    } else if constexpr (D == 256) {
        // (the 128-row tile fills its 256 registers: the second copy of the exponentials that the lagging reference
        // needs spilled 20 bytes more and ran 9 % slower, so it keeps the exact maximum per step)
        if (variant == 6) return launch_one16<D, 1, 8, 1, 32, 2, D, 1>(p, s);
        if (variant == 3 || variant == 4) return launch_one16<D, 1, 2, 2, 32, 1>(p, s);
        return launch_one16<D, 1, 4, 1, 32, 2, D, 1>(p, s);
    } else
    switch (variant) {
        case 1: return launch_one16<D, 1, 4, 1, 64, 2>(p, s);
        case 2:
            if constexpr (D == 128) return launch_one16<D, 1, 4, 1, 64, 2>(p, s);   // two query groups would spill
            // 128-key tiles (78 KB of LDS; registers allow two blocks per CU anyway) and the K fragments of the next
            // step requested early: +2-4 % over 64-key tiles (measured in one process: 893 against 874 TFLOP/s at
            // n = 16384, 846 against 818 at 8192); at d = 128 the early request measured -1 % and is not used
            else return launch_one16<D, 2, 4, 1, 128, 2, D, 3>(p, s);
        case 3:
            if constexpr (D == 128) return launch_one16<D, 1, 2, 2, 32, 2>(p, s);
            else return launch_one16<D, 1, 1, 4, 32, 2>(p, s);
        case 4: return launch_one16<D, 1, 2, 2, 32, 2>(p, s);
        case 5:
            if constexpr (D <= 64) return launch_one16<D, 2, 4, 1, 64, 2, D, 0>(p, s);
            else return (int)hipErrorInvalidValue;
        case 6:
            if constexpr (D == 128) return launch_one16<D, 1, 8, 1, 64, 2>(p, s);
            else return (int)hipErrorInvalidValue;
        default: return (int)hipErrorInvalidValue;
    }
}

int launch_fwd_mfma16(const FwdParams &p, int d, int variant, hipStream_t s, const char **name) {
    if (name) *name = mfma16_variant_name(variant);
    if (d == 32) return launch_variant16<32>(p, variant, s);
    if (d == 64) return launch_variant16<64>(p, variant, s);
    if (d == 128) return launch_variant16<128>(p, variant, s);
    if (d == 96) return launch_variant16<96>(p, variant, s);
    if (d == 256) return launch_variant16<256>(p, variant, s);
    return (int)hipErrorInvalidValue;
}

}  // namespace elsa
