// 16-bit storage, all four layouts: 128 x 128 tile kernels built on the 16x16x32 MFMA (mid-size problems).
#include "variant16.h"

namespace peak {

static const Variant rows_mf16s[] = {
    // 64x64 per wave as 4 x 4 blocks of 16x16, three A stages and two B stages in 80 KB: two workgroups per CU
    TILED_MF16("bf16_m128x128w4a3_nt", DT_BF16, 0, 0, 128, 2),
    TILED_MF16("f16_m128x128w4a3_nt", DT_F16, 0, 0, 128, 2),
    TILED_MF16("bf16_m128x128w4a3_nn", DT_BF16, 0, 1, 128, 2),
    TILED_MF16("f16_m128x128w4a3_nn", DT_F16, 0, 1, 128, 2),
    TILED_MF16("bf16_m128x128w4a3_tt", DT_BF16, 1, 0, 128, 2),
    TILED_MF16("f16_m128x128w4a3_tt", DT_F16, 1, 0, 128, 2),
    TILED_MF16("bf16_m128x128w4a3_tn", DT_BF16, 1, 1, 128, 2),
    TILED_MF16("f16_m128x128w4a3_tn", DT_F16, 1, 1, 128, 2),
};

PEAK_VARIANT_GROUP(variants_mf16s, rows_mf16s)

}  // namespace peak
