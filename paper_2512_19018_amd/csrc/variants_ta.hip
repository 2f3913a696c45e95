// A stored K x M ("_t?"): staged directly as [k][m] rows.
#include "variant.h"

namespace peak {

static const Variant rows_ta[] = {
    TILED_ATR("bf16_t256x256w8_tt", DT_BF16, 256, 256, 128, 2, 4, 2, 0),
    TILED_ATR("f16_t256x256w8_tt", DT_F16, 256, 256, 128, 2, 4, 2, 0),
    TILED_ATR("bf16_t256x256w8_tn", DT_BF16, 256, 256, 128, 2, 4, 2, 1),
    TILED_ATR("f16_t256x256w8_tn", DT_F16, 256, 256, 128, 2, 4, 2, 1),
    TILED_ATR("bf16_t128x128w4_tt", DT_BF16, 128, 128, 128, 2, 2, 2, 0),
    TILED_ATR("f16_t128x128w4_tt", DT_F16, 128, 128, 128, 2, 2, 2, 0),
    TILED_ATR("bf16_t128x128w4_tn", DT_BF16, 128, 128, 128, 2, 2, 2, 1),
    TILED_ATR("f16_t128x128w4_tn", DT_F16, 128, 128, 128, 2, 2, 2, 1),
    TILED_ATR("f32_t128x128w4_tt", DT_F32, 128, 128, 128, 2, 2, 2, 0),
    TILED_ATR("f32_t128x128w4_tn", DT_F32, 128, 128, 128, 2, 2, 2, 1),
    TILED_ATR("f32_t256x128w8_tt", DT_F32, 256, 128, 128, 4, 2, 2, 0),
    TILED_ATR("f32_t256x128w8_tn", DT_F32, 256, 128, 128, 4, 2, 2, 1),
};

PEAK_VARIANT_GROUP(variants_ta, rows_ta)

}  // namespace peak
