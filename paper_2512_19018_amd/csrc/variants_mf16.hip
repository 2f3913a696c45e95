// 16-bit storage, both operands running along K ("_nt"): kernels built on the 16x16x32 MFMA.
#include "variant.h"
#include "gemm16_device.h"

namespace peak {

template <class C>
static int launch_gemm16(const GemmArgs &a, unsigned grid, void *stream)
{
    // K ending inside a K tile takes the instantiation that can zero-fill the tail
    if (a.K % C::BK != 0) hipLaunchKernelGGL((gemm16_kernel<C, true>), dim3(grid), dim3(C::NT), 0, (hipStream_t)stream, a);
    else hipLaunchKernelGGL((gemm16_kernel<C, false>), dim3(grid), dim3(C::NT), 0, (hipStream_t)stream, a);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

// AKM: A stored K x M, staged as [k][m] rows; BKN: B stored K x N, staged as [k][n] rows
#define TILED_MF16(NAME, DT, AKM, BKN)                                                                 \
    {NAME, KIND_TILED, DT, AKM, BKN, 1, 256, 256, 64, 256, 2,                                          \
     Cfg16<DT, AKM != 0, BKN != 0>::LDS_BYTES, 0, &launch_gemm16<Cfg16<DT, AKM != 0, BKN != 0>>, BKN, AKM, 0, 0, 1}

static const Variant rows_mf16[] = {
    // one wave per SIMD, 128x128 per wave as 8 x 8 blocks of 16x16, three A stages and two B stages
    TILED_MF16("bf16_m256x256w4a3_nt", DT_BF16, 0, 0),
    TILED_MF16("f16_m256x256w4a3_nt", DT_F16, 0, 0),
    TILED_MF16("bf16_m256x256w4a3_nn", DT_BF16, 0, 1),
    TILED_MF16("f16_m256x256w4a3_nn", DT_F16, 0, 1),
    TILED_MF16("bf16_m256x256w4a3_tt", DT_BF16, 1, 0),
    TILED_MF16("f16_m256x256w4a3_tt", DT_F16, 1, 0),
    TILED_MF16("bf16_m256x256w4a3_tn", DT_BF16, 1, 1),
    TILED_MF16("f16_m256x256w4a3_tn", DT_F16, 1, 1),
};

PEAK_VARIANT_GROUP(variants_mf16, rows_mf16)

}  // namespace peak
