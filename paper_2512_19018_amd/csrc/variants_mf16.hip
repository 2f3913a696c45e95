// 16-bit storage, all four layouts: 256 x 256 tile kernels built on the 16x16x32 MFMA.
#include "variant16.h"

namespace peak {

static const Variant rows_mf16[] = {
    // one wave per SIMD, 128x128 per wave as 8 x 8 blocks of 16x16, three A stages and two B stages
    TILED_MF16("bf16_m256x256w4a3_nt", DT_BF16, 0, 0, 256, 2),
    TILED_MF16("f16_m256x256w4a3_nt", DT_F16, 0, 0, 256, 2),
    TILED_MF16("bf16_m256x256w4a3_nn", DT_BF16, 0, 1, 256, 2),
    TILED_MF16("f16_m256x256w4a3_nn", DT_F16, 0, 1, 256, 2),
    TILED_MF16("bf16_m256x256w4a3_tt", DT_BF16, 1, 0, 256, 2),
    TILED_MF16("f16_m256x256w4a3_tt", DT_F16, 1, 0, 256, 2),
    TILED_MF16("bf16_m256x256w4a3_tn", DT_BF16, 1, 1, 256, 2),
    TILED_MF16("f16_m256x256w4a3_tn", DT_F16, 1, 1, 256, 2),
};

PEAK_VARIANT_GROUP(variants_mf16, rows_mf16)

}  // namespace peak
