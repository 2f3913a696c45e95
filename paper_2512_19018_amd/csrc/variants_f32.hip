// fp32, A along K: A direct; B through registers ("_d", either layout) or directly
// as [k][n] rows ("_t": no transposition needed, one float per lane and MFMA).
#include "variant.h"

namespace peak {

static const Variant rows_f32[] = {
    TILED("f32_d128x128w4_nt", DT_F32, 128, 128, 128, 2, 2, 2, false, false, true),
    TILED("f32_d128x128w4s3_nt", DT_F32, 128, 128, 128, 2, 2, 3, false, false, true),
    TILED("f32_d128x128w4_nn", DT_F32, 128, 128, 128, 2, 2, 2, false, true, true),
    TILED("f32_d128x128w4s3_nn", DT_F32, 128, 128, 128, 2, 2, 3, false, true, true),
    TILED("f32_d256x128w8_nn", DT_F32, 256, 128, 128, 4, 2, 2, false, true, true),
    TILED("f32_d256x128w8s3_nn", DT_F32, 256, 128, 128, 4, 2, 3, false, true, true),
    TILED_TR("f32_t128x128w4_nn", DT_F32, 128, 128, 128, 2, 2, 2),
    TILED_TR("f32_t128x128w4s3_nn", DT_F32, 128, 128, 128, 2, 2, 3),
    TILED_TR_AG("f32_t128x128w4g_nn", 128, 128),
    TILED_TR("f32_t256x128w8_nn", DT_F32, 256, 128, 128, 4, 2, 2),
    TILED_TR("f32_t256x128w8s3_nn", DT_F32, 256, 128, 128, 4, 2, 3),
    TILED_TR("f32_t256x128w4_nn", DT_F32, 256, 128, 128, 2, 2, 2),
    TILED_TR("f32_t128x64w4_nn", DT_F32, 128, 64, 128, 2, 2, 2),
    // one wave per SIMD, 128x128 per wave (a quarter of the LDS fragment traffic per multiply-add of
    // 64x64 wave tiles), accumulators in AGPRs, three A stages
    TILED_AX("f32_d256x256w4a3_nt", DT_F32, 256, 256, 128, 2, 2, 2, 1),
    TILED_AX_TR("f32_t256x256w4a3_nn", DT_F32, 256, 256, 128, 2, 2, 2, 1),
};

PEAK_VARIANT_GROUP(variants_f32, rows_f32)

}  // namespace peak
