// 16-bit storage, all four layouts: the 128 x 128 tile of the 16x16x32 MFMA kernels with loads four K tiles ahead.
#include "variant16.h"

namespace peak {

static const Variant rows_mf16d[] = {
    // the same tile with five A stages and four B stages (144 KB: one workgroup per CU), loads four K tiles ahead:
    // for problems of at most one tile per CU, where nothing else covers a load's latency
    TILED_MF16("bf16_m128x128w4a5_nt", DT_BF16, 0, 0, 128, 4),
    TILED_MF16("f16_m128x128w4a5_nt", DT_F16, 0, 0, 128, 4),
    TILED_MF16("bf16_m128x128w4a5_nn", DT_BF16, 0, 1, 128, 4),
    TILED_MF16("f16_m128x128w4a5_nn", DT_F16, 0, 1, 128, 4),
    TILED_MF16("bf16_m128x128w4a5_tt", DT_BF16, 1, 0, 128, 4),
    TILED_MF16("f16_m128x128w4a5_tt", DT_F16, 1, 0, 128, 4),
    TILED_MF16("bf16_m128x128w4a5_tn", DT_BF16, 1, 1, 128, 4),
    TILED_MF16("f16_m128x128w4a5_tn", DT_F16, 1, 1, 128, 4),
};

PEAK_VARIANT_GROUP(variants_mf16d, rows_mf16d)

}  // namespace peak
