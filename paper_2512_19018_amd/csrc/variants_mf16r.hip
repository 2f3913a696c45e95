// 16-bit storage, all four layouts: 256 x 128 tile kernels built on the 16x16x32 MFMA.
#include "variant16.h"

namespace peak {

static const Variant rows_mf16r[] = {
    // 128x64 per wave as 8 x 4 blocks of 16x16, three A stages (32 KB) and two B stages (16 KB): 128 KB, one workgroup per CU
    TILED_MF16_MN("bf16_m256x128w4a3_nt", DT_BF16, 0, 0, 256, 128, 2),
    TILED_MF16_MN("f16_m256x128w4a3_nt", DT_F16, 0, 0, 256, 128, 2),
    TILED_MF16_MN("bf16_m256x128w4a3_nn", DT_BF16, 0, 1, 256, 128, 2),
    TILED_MF16_MN("f16_m256x128w4a3_nn", DT_F16, 0, 1, 256, 128, 2),
    TILED_MF16_MN("bf16_m256x128w4a3_tt", DT_BF16, 1, 0, 256, 128, 2),
    TILED_MF16_MN("f16_m256x128w4a3_tt", DT_F16, 1, 0, 256, 128, 2),
    TILED_MF16_MN("bf16_m256x128w4a3_tn", DT_BF16, 1, 1, 256, 128, 2),
    TILED_MF16_MN("f16_m256x128w4a3_tn", DT_F16, 1, 1, 256, 128, 2),
    // (a form with three stages of each operand, all loads behind the tile's barrier, measured no better: bf16
    // 2048x4096x4096 57.4 us against 55.8)
};

PEAK_VARIANT_GROUP(variants_mf16r, rows_mf16r)

}  // namespace peak
