// 16-bit storage, all four layouts: 128 x 128 tile kernels on the 16x16x32 MFMA with 128 k per stage.
#include "variant16.h"

namespace peak {

static const Variant rows_mf16k[] = {
    // 64x64 per wave, three A stages and two B stages of 32 KB (160 KB: one workgroup per CU), four k-steps per K tile
    TILED_MF16_K("bf16_m128x128k128w4a3_nt", DT_BF16, 0, 0, 128, 128, 2, 128),
    TILED_MF16_K("f16_m128x128k128w4a3_nt", DT_F16, 0, 0, 128, 128, 2, 128),
    TILED_MF16_K("bf16_m128x128k128w4a3_nn", DT_BF16, 0, 1, 128, 128, 2, 128),
    TILED_MF16_K("f16_m128x128k128w4a3_nn", DT_F16, 0, 1, 128, 128, 2, 128),
    TILED_MF16_K("bf16_m128x128k128w4a3_tt", DT_BF16, 1, 0, 128, 128, 2, 128),
    TILED_MF16_K("f16_m128x128k128w4a3_tt", DT_F16, 1, 0, 128, 128, 2, 128),
    TILED_MF16_K("bf16_m128x128k128w4a3_tn", DT_BF16, 1, 1, 128, 128, 2, 128),
    TILED_MF16_K("f16_m128x128k128w4a3_tn", DT_F16, 1, 1, 128, 128, 2, 128),
};

PEAK_VARIANT_GROUP(variants_mf16k, rows_mf16k)

}  // namespace peak
