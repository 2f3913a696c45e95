// Kernel variant table: one row per instantiation of the kernel templates (the
// tuning parameters of the paper's Section 3.1: tile shape, waves, stages,
// staging kind).  The rows are defined in several translation units, one per
// group of variants, so that the groups compile in parallel; peak_gemm.hip
// joins them into one table.
#pragma once

#include <hip/hip_runtime.h>

#include "gemm_device.h"
#include "planner.h"

namespace peak {

// one per translation unit
VariantGroup variants_general();
VariantGroup variants_bf16_nt();
VariantGroup variants_f16_nt();
VariantGroup variants_bf16_nn();
VariantGroup variants_f16_nn();
VariantGroup variants_f32();
VariantGroup variants_ta();
VariantGroup variants_skinny();
VariantGroup variants_mf16();
VariantGroup variants_mf16s();
VariantGroup variants_mf16d();
VariantGroup variants_mf16r();
VariantGroup variants_mf16k();

template <class C>
static int launch_gemm(const GemmArgs &a, unsigned grid, void *stream)
{
    hipLaunchKernelGGL((gemm_kernel<C>), dim3(grid), dim3(C::NT), 0, (hipStream_t)stream, a);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

#define PEAK_BK(DT, RB) ((RB) / ((DT) == DT_F32 ? 4 : 2))

// both operands handled by the template's own flags
#define TILED(NAME, DT, BM, BN, RB, WMW, WNW, NS, AT, BT, DIR)                                         \
    {NAME, KIND_TILED, DT, AT, BT, DIR, BM, BN, PEAK_BK(DT, RB), WMW * WNW * 64, NS,                   \
     Cfg<DT, BM, BN, RB, WMW, WNW, NS, AT, BT, DIR>::LDS_BYTES, 0,                                     \
     &launch_gemm<Cfg<DT, BM, BN, RB, WMW, WNW, NS, AT, BT, DIR>>, 0, 0, 0, 0}

// the same, reachable through the force bits only
#define TILED_SWEEP(NAME, DT, BM, BN, RB, WMW, WNW, NS, AT, BT, DIR)                                   \
    {NAME, KIND_TILED, DT, AT, BT, DIR, BM, BN, PEAK_BK(DT, RB), WMW * WNW * 64, NS,                   \
     Cfg<DT, BM, BN, RB, WMW, WNW, NS, AT, BT, DIR>::LDS_BYTES, 0,                                     \
     &launch_gemm<Cfg<DT, BM, BN, RB, WMW, WNW, NS, AT, BT, DIR>>, 0, 0, 1, 0}

// AX extra A stages (both operands along K)
#define TILED_AX(NAME, DT, BM, BN, RB, WMW, WNW, NS, AX)                                              \
    {NAME, KIND_TILED, DT, 0, 0, 1, BM, BN, PEAK_BK(DT, RB), WMW * WNW * 64, NS,                       \
     Cfg<DT, BM, BN, RB, WMW, WNW, NS, false, false, true, AX>::LDS_BYTES, 0,                          \
     &launch_gemm<Cfg<DT, BM, BN, RB, WMW, WNW, NS, false, false, true, AX>>, 0, 0, 0, 0}

// AX extra A stages, B kept as [k][n] rows
#define TILED_AX_TR(NAME, DT, BM, BN, RB, WMW, WNW, NS, AX)                                           \
    {NAME, KIND_TILED, DT, 0, 1, 1, BM, BN, PEAK_BK(DT, RB), WMW * WNW * 64, NS,                       \
     Cfg<DT, BM, BN, RB, WMW, WNW, NS, false, true, true, AX, true>::LDS_BYTES, 0,                     \
     &launch_gemm<Cfg<DT, BM, BN, RB, WMW, WNW, NS, false, true, true, AX, true>>, 1, 0, 0, 0}

// B kept as [k][n] rows
#define TILED_TR(NAME, DT, BM, BN, RB, WMW, WNW, NS)                                                   \
    {NAME, KIND_TILED, DT, 0, 1, 1, BM, BN, PEAK_BK(DT, RB), WMW * WNW * 64, NS,                       \
     Cfg<DT, BM, BN, RB, WMW, WNW, NS, false, true, true, 0, true>::LDS_BYTES, 0,                      \
     &launch_gemm<Cfg<DT, BM, BN, RB, WMW, WNW, NS, false, true, true, 0, true>>, 1, 0, 0, 0}

// fp32, B kept as [k][n] rows, 128x128 tile of four 64x64 wave tiles, hand-scheduled loop
#define TILED_TR_AG(NAME, BM, BN)                                                                      \
    {NAME, KIND_TILED, DT_F32, 0, 1, 1, BM, BN, PEAK_BK(DT_F32, 128), 256, 2,                          \
     Cfg<DT_F32, BM, BN, 128, 2, 2, 2, false, true, true, 0, true, false, false, true>::LDS_BYTES, 0,  \
     &launch_gemm<Cfg<DT_F32, BM, BN, 128, 2, 2, 2, false, true, true, 0, true, false, false, true>>, 1, 0, 0, 0}

// A stored K x M staged directly as [k][m] rows; B either along K ("_tt") or [k][n] rows as well ("_tn")
#define TILED_ATR(NAME, DT, BM, BN, RB, WMW, WNW, NS, BTR)                                             \
    {NAME, KIND_TILED, DT, 1, BTR, 1, BM, BN, PEAK_BK(DT, RB), WMW * WNW * 64, NS,                     \
     Cfg<DT, BM, BN, RB, WMW, WNW, NS, true, BTR != 0, true, 0, BTR != 0, false, true>::LDS_BYTES, 0,  \
     &launch_gemm<Cfg<DT, BM, BN, RB, WMW, WNW, NS, true, BTR != 0, true, 0, BTR != 0, false, true>>, BTR, 1, 0, 0}

// alternating main loop (sweeps only)
#define TILED_PP(NAME, DT, BM, BN, RB, WMW, WNW, NS, TR)                                              \
    {NAME, KIND_TILED, DT, 0, TR, 1, BM, BN, PEAK_BK(DT, RB), WMW * WNW * 64, NS,                      \
     Cfg<DT, BM, BN, RB, WMW, WNW, NS, false, TR != 0, true, 0, TR != 0, true>::LDS_BYTES, 0,          \
     &launch_gemm<Cfg<DT, BM, BN, RB, WMW, WNW, NS, false, TR != 0, true, 0, TR != 0, true>>, TR, 0, 1, 0}

// Layout suffix of the names: first letter is A (n: runs along K, t: stored K x M),
// second is B as stored (t: N x K, runs along K; n: K x N).  So "_nt" is transA=0,
// transB=1: both operands K-contiguous.
#define TILED_LAYOUTS(NAME, DT, BM, BN, RB, WMW, WNW, NS)                                              \
    TILED(NAME "_nt", DT, BM, BN, RB, WMW, WNW, NS, false, false, false),                             \
    TILED(NAME "_nn", DT, BM, BN, RB, WMW, WNW, NS, false, true, false),                              \
    TILED(NAME "_tt", DT, BM, BN, RB, WMW, WNW, NS, true, false, false),                              \
    TILED(NAME "_tn", DT, BM, BN, RB, WMW, WNW, NS, true, true, false)

#define PEAK_VARIANT_GROUP(FN, ROWS)                                                                   \
    VariantGroup FN() { return VariantGroup{ROWS, (int)(sizeof(ROWS) / sizeof(ROWS[0]))}; }

}  // namespace peak
