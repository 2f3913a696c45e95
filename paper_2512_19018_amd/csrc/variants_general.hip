// Register-staged tiles: any alignment, any K, all four layouts.
#include "variant.h"

namespace peak {

static const Variant rows_general[] = {
    TILED_LAYOUTS("f32_r128x128", DT_F32, 128, 128, 128, 2, 2, 2),
    TILED_LAYOUTS("f16_r128x128", DT_F16, 128, 128, 128, 2, 2, 2),
    TILED_LAYOUTS("bf16_r128x128", DT_BF16, 128, 128, 128, 2, 2, 2),
    TILED_LAYOUTS("f32_r64x64", DT_F32, 64, 64, 128, 2, 2, 2),
    TILED_LAYOUTS("f16_r64x64", DT_F16, 64, 64, 128, 2, 2, 2),
    TILED_LAYOUTS("bf16_r64x64", DT_BF16, 64, 64, 128, 2, 2, 2),
};

PEAK_VARIANT_GROUP(variants_general, rows_general)

}  // namespace peak
