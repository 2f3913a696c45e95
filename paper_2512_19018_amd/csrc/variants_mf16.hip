// 16-bit storage, both operands running along K ("_nt"): kernels built on the 16x16x32 MFMA.
#include "variant.h"
#include "gemm16_device.h"

namespace peak {

template <class C>
static hipError_t launch_gemm16(const GemmArgs &a, dim3 grid, hipStream_t s)
{
    hipLaunchKernelGGL((gemm16_kernel<C>), grid, dim3(C::NT), 0, s, a);
    return hipGetLastError();
}

#define TILED_MF16(NAME, DT)                                                                           \
    {NAME, KIND_TILED, DT, 0, 0, 1, Cfg16<DT>::BM, Cfg16<DT>::BN, Cfg16<DT>::BK, Cfg16<DT>::NT, Cfg16<DT>::NSB,   \
     Cfg16<DT>::LDS_BYTES, 0, &launch_gemm16<Cfg16<DT>>, 0, 0, 0, 0, 1}

static const Variant rows_mf16[] = {
    // one wave per SIMD, 128x128 per wave as 8 x 8 blocks of 16x16, three A stages and two B stages
    TILED_MF16("bf16_m256x256w4a3_nt", DT_BF16),
    TILED_MF16("f16_m256x256w4a3_nt", DT_F16),
};

PEAK_VARIANT_GROUP(variants_mf16, rows_mf16)

}  // namespace peak
