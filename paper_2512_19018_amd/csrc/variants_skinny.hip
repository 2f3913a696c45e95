// Streaming kernels for M <= 16 with both operands along K: B is read once.
#include "variant.h"
#include "skinny_device.h"

namespace peak {

template <class C>
static hipError_t launch_skinny(const GemmArgs &a, dim3 grid, hipStream_t s)
{
    hipLaunchKernelGGL((skinny_kernel<C>), grid, dim3(C::NT), 0, s, a);
    return hipGetLastError();
}

template <class C>
static hipError_t launch_skinny_reg(const GemmArgs &a, dim3 grid, hipStream_t s)
{
    hipLaunchKernelGGL((skinny_reg_kernel<C>), grid, dim3(C::NT), 0, s, a);
    return hipGetLastError();
}

#define SKINNY(NAME, DT, BN, KSTEP, NS, RANK)                                                          \
    {NAME, KIND_SKINNY, DT, 0, 0, 1, 16, BN, KSTEP, SkinnyCfg<DT, BN, KSTEP, NS>::NT, NS,              \
     SkinnyCfg<DT, BN, KSTEP, NS>::LDS_BYTES, 16, &launch_skinny<SkinnyCfg<DT, BN, KSTEP, NS>>, 0, 0, RANK == 0, RANK}

#define SKINNY_REG(NAME, DT, DEPTH, WAVES, RANK)                                                       \
    {NAME, KIND_SKINNY_REG, DT, 0, 0, 1, 16, 16, 64, WAVES * 64, DEPTH, 0, 16,                         \
     &launch_skinny_reg<SkinnyRegCfg<DT, DEPTH, WAVES>>, 0, 0, RANK == 0, RANK}

static const Variant rows_skinny[] = {
    // LDS ring of BN rows x KSTEP ...
    SKINNY("bf16_skinny16s3_nt", DT_BF16, 64, 128, 3, 0),
    SKINNY("f16_skinny16s3_nt", DT_F16, 64, 128, 3, 0),
    SKINNY("bf16_skinny32k512s3_nt", DT_BF16, 32, 512, 3, 0),
    SKINNY("f16_skinny32k512s3_nt", DT_F16, 32, 512, 3, 0),
    SKINNY("bf16_skinny64k256s3_nt", DT_BF16, 64, 256, 3, 0),
    SKINNY("f16_skinny64k256s3_nt", DT_F16, 64, 256, 3, 0),
    // deeper rings of shorter stages: more of the stream in flight per CU for the same 160 KB
    SKINNY("bf16_skinny64k256s4_nt", DT_BF16, 64, 256, 4, 0),
    SKINNY("f16_skinny64k256s4_nt", DT_F16, 64, 256, 4, 0),
    SKINNY("bf16_skinny64k128s8_nt", DT_BF16, 64, 128, 8, 0),
    SKINNY("f16_skinny64k128s8_nt", DT_F16, 64, 128, 8, 0),
    // long row runs through LDS: the selector's first choice wherever K is a multiple of 512
    SKINNY("bf16_skinny64k512s2_nt", DT_BF16, 64, 512, 2, 2),
    SKINNY("f16_skinny64k512s2_nt", DT_F16, 64, 512, 2, 2),
    // ... or straight into registers (no LDS, no barriers): the second choice, for other K
    SKINNY_REG("bf16_skinnyreg_d8_nt", DT_BF16, 8, 4, 1),
    SKINNY_REG("f16_skinnyreg_d8_nt", DT_F16, 8, 4, 1),
};

PEAK_VARIANT_GROUP(variants_skinny, rows_skinny)

}  // namespace peak
