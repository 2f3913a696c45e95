// Streaming kernels for M <= 64 with A along K and B either along K or stored K x N: B is read once.
#include "variant.h"
#include "skinny_device.h"

namespace peak {

template <class C>
static int launch_skinny(const GemmArgs &a, unsigned grid, void *stream)
{
    hipLaunchKernelGGL((skinny_kernel<C>), dim3(grid), dim3(C::NT), 0, (hipStream_t)stream, a);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

template <class C>
static int launch_skinny_reg(const GemmArgs &a, unsigned grid, void *stream)
{
    hipLaunchKernelGGL((skinny_reg_kernel<C>), dim3(grid), dim3(C::NT), 0, (hipStream_t)stream, a);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

template <class C>
static int launch_skinny_kn(const GemmArgs &a, unsigned grid, void *stream)
{
    hipLaunchKernelGGL((skinny_kn_kernel<C>), dim3(grid), dim3(C::NT), 0, (hipStream_t)stream, a);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

// B stored K x N, kept as [k][n] rows
#define SKINNY_KN(NAME, DT, NS, MBLK, RANK)                                                            \
    {NAME, KIND_SKINNY, DT, 0, 1, 1, 16 * MBLK, SkinnyKnCfg<DT, NS, MBLK>::BN, SkinnyKnCfg<DT, NS, MBLK>::KSTEP,        \
     SkinnyKnCfg<DT, NS, MBLK>::NT, NS, SkinnyKnCfg<DT, NS, MBLK>::LDS_BYTES, 16 * MBLK,               \
     &launch_skinny_kn<SkinnyKnCfg<DT, NS, MBLK>>, 1, 0, RANK == 0, RANK}

#define SKINNY(NAME, DT, BN, KSTEP, NS, RANK)                                                          \
    {NAME, KIND_SKINNY, DT, 0, 0, 1, 16, BN, KSTEP, SkinnyCfg<DT, BN, KSTEP, NS>::NT, NS,              \
     SkinnyCfg<DT, BN, KSTEP, NS>::LDS_BYTES, 16, &launch_skinny<SkinnyCfg<DT, BN, KSTEP, NS>>, 0, 0, RANK == 0, RANK}

// MBLK blocks of 16 rows of the M x K operand
#define SKINNY_M(NAME, DT, BN, KSTEP, NS, MBLK, RANK)                                                  \
    {NAME, KIND_SKINNY, DT, 0, 0, 1, 16 * MBLK, BN, KSTEP, SkinnyCfg<DT, BN, KSTEP, NS, MBLK>::NT, NS, \
     SkinnyCfg<DT, BN, KSTEP, NS, MBLK>::LDS_BYTES, 16 * MBLK,                                         \
     &launch_skinny<SkinnyCfg<DT, BN, KSTEP, NS, MBLK>>, 0, 0, RANK == 0, RANK}

// ... with the loop pipelined across the stage's barrier (KW waves per 16 rows)
#define SKINNY_MP(NAME, DT, BN, KSTEP, NS, MBLK, KW, RANK)                                             \
    {NAME, KIND_SKINNY, DT, 0, 0, 1, 16 * MBLK, BN, KSTEP, SkinnyCfg<DT, BN, KSTEP, NS, MBLK, KW, 1>::NT, NS, \
     SkinnyCfg<DT, BN, KSTEP, NS, MBLK, KW, 1>::LDS_BYTES, 16 * MBLK,                                  \
     &launch_skinny<SkinnyCfg<DT, BN, KSTEP, NS, MBLK, KW, 1>>, 0, 0, RANK == 0, RANK}

#define SKINNY_REG(NAME, DT, DEPTH, WAVES, RANK)                                                       \
    {NAME, KIND_SKINNY_REG, DT, 0, 0, 1, 16, 16, 64, WAVES * 64, DEPTH, 0, 16,                         \
     &launch_skinny_reg<SkinnyRegCfg<DT, DEPTH, WAVES>>, 0, 0, RANK == 0, RANK}

static const Variant rows_skinny[] = {
    // LDS ring of BN rows x KSTEP ...
    // 64 rows x 128 k, three stages: the selector's usual choice (K a multiple of 128)
    SKINNY("bf16_skinny16s3_nt", DT_BF16, 64, 128, 3, 2),
    SKINNY("f16_skinny16s3_nt", DT_F16, 64, 128, 3, 2),
    // (the loop pipelined across the barrier, as for fp32 below, changes nothing here: 86.0 us against 85.9)
    SKINNY("bf16_skinny32k512s3_nt", DT_BF16, 32, 512, 3, 0),
    SKINNY("f16_skinny32k512s3_nt", DT_F16, 32, 512, 3, 0),
    SKINNY("bf16_skinny64k256s3_nt", DT_BF16, 64, 256, 3, 0),
    SKINNY("f16_skinny64k256s3_nt", DT_F16, 64, 256, 3, 0),
    // deeper rings of shorter stages: more of the stream in flight per CU for the same 160 KB
    SKINNY("bf16_skinny64k256s4_nt", DT_BF16, 64, 256, 4, 0),
    SKINNY("f16_skinny64k256s4_nt", DT_F16, 64, 256, 4, 0),
    SKINNY("bf16_skinny64k128s8_nt", DT_BF16, 64, 128, 8, 0),
    SKINNY("f16_skinny64k128s8_nt", DT_F16, 64, 128, 8, 0),
    // 128 rows per workgroup: the M x K operand, which every workgroup reads in full, crosses the L1 half as often
    // (first choice when N / 128 workgroups fill the chip without a K split: f16 16x28672x8192 74.6 us against 82.4)
    SKINNY("bf16_skinny128k256s2_nt", DT_BF16, 128, 256, 2, 3),
    SKINNY("f16_skinny128k256s2_nt", DT_F16, 128, 256, 2, 3),
    SKINNY("bf16_skinny128k128s3_nt", DT_BF16, 128, 128, 3, 0),
    SKINNY("f16_skinny128k128s3_nt", DT_F16, 128, 128, 3, 0),
    // (256 rows per workgroup, 16 waves, measured slower than 128: bf16 16x28672x8192 81.3 us against 74.5)
    // long row runs through LDS
    SKINNY("bf16_skinny64k512s2_nt", DT_BF16, 64, 512, 2, 0),
    SKINNY("f16_skinny64k512s2_nt", DT_F16, 64, 512, 2, 0),
    // ... or straight into registers (no LDS, no barriers): the second choice, for other K
    SKINNY_REG("bf16_skinnyreg_d8_nt", DT_BF16, 8, 4, 1),
    SKINNY_REG("f16_skinnyreg_d8_nt", DT_F16, 8, 4, 1),
    // fp32: 64 k per stage row (256 bytes), 16x16x4 MFMA
    SKINNY("f32_skinny_m16n64k64s3_nt", DT_F32, 64, 64, 3, 2),
    SKINNY("f32_skinny_m16n128k64s3_nt", DT_F32, 128, 64, 3, 3),
    SKINNY("f32_skinny_m16n64k128s3_nt", DT_F32, 64, 128, 3, 0),
    // 16 < M <= 32 and 32 < M <= 64: two or four 16-row blocks of the M x K operand per stage.  The rows come after
    // the single-block ones, so that the selector's "first that fits" takes the fewest blocks that hold M.
    SKINNY_M("bf16_skinny_m32n64k128s3_nt", DT_BF16, 64, 128, 3, 2, 2),
    SKINNY_M("f16_skinny_m32n64k128s3_nt", DT_F16, 64, 128, 3, 2, 2),
    SKINNY_M("bf16_skinny_m32n128k128s3_nt", DT_BF16, 128, 128, 3, 2, 3),
    SKINNY_M("f16_skinny_m32n128k128s3_nt", DT_F16, 128, 128, 3, 2, 3),
    // fp32 with several blocks is bound by the MFMAs: two waves per 16 rows and the loop pipelined across the stage's
    // barrier (64x16384x8192: 154.6 us against 174; 48x28672x8192: 275 against 314; 32x16384x8192: 93.9 against 104.7)
    SKINNY_MP("f32_skinny_m32n64k64s3w8p_nt", DT_F32, 64, 64, 3, 2, 2, 2),
    SKINNY_MP("f32_skinny_m32n64k64s3p_nt", DT_F32, 64, 64, 3, 2, 1, 0),
    SKINNY_M("f32_skinny_m32n64k64s3_nt", DT_F32, 64, 64, 3, 2, 0),
    SKINNY_M("bf16_skinny_m64n64k128s3_nt", DT_BF16, 64, 128, 3, 4, 2),
    SKINNY_M("f16_skinny_m64n64k128s3_nt", DT_F16, 64, 128, 3, 4, 2),
    SKINNY_M("bf16_skinny_m64n128k128s3_nt", DT_BF16, 128, 128, 3, 4, 3),
    SKINNY_M("f16_skinny_m64n128k128s3_nt", DT_F16, 128, 128, 3, 4, 3),
    SKINNY_MP("f32_skinny_m64n64k64s3w8p_nt", DT_F32, 64, 64, 3, 4, 2, 2),
    SKINNY_MP("f32_skinny_m64n64k64s3p_nt", DT_F32, 64, 64, 3, 4, 1, 0),
    SKINNY_M("f32_skinny_m64n64k64s3_nt", DT_F32, 64, 64, 3, 4, 0),
    // (more blocks, M up to 128 or 256, measured no better than the tiled kernels: the M x K operand, re-read by
    // every workgroup from the L2, then outweighs B: bf16 128x28672x8192 111 us against 114, 256x... behind)
    // B stored K x N: 512 bytes of every k-row per workgroup, 128 bytes of K per stage
    SKINNY_KN("bf16_skinny_m16n256k64s4_nn", DT_BF16, 4, 1, 2),
    SKINNY_KN("f16_skinny_m16n256k64s4_nn", DT_F16, 4, 1, 2),
    SKINNY_KN("f32_skinny_m16n128k32s6_nn", DT_F32, 6, 1, 2),
    SKINNY_KN("bf16_skinny_m16n256k64s3_nn", DT_BF16, 3, 1, 0),
    SKINNY_KN("f16_skinny_m16n256k64s3_nn", DT_F16, 3, 1, 0),
    SKINNY_KN("f32_skinny_m16n128k32s8_nn", DT_F32, 8, 1, 0),
    SKINNY_KN("bf16_skinny_m32n256k64s4_nn", DT_BF16, 4, 2, 2),
    SKINNY_KN("f16_skinny_m32n256k64s4_nn", DT_F16, 4, 2, 2),
    SKINNY_KN("f32_skinny_m32n128k32s6_nn", DT_F32, 6, 2, 2),
    SKINNY_KN("bf16_skinny_m64n256k64s4_nn", DT_BF16, 4, 4, 2),
    SKINNY_KN("f16_skinny_m64n256k64s4_nn", DT_F16, 4, 4, 2),
    SKINNY_KN("f32_skinny_m64n128k32s6_nn", DT_F32, 6, 4, 2),
};

PEAK_VARIANT_GROUP(variants_skinny, rows_skinny)

}  // namespace peak
