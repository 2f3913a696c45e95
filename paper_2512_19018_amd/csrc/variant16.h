// Launch of the 16x16x32-MFMA kernels and the macro for their rows of the variant table.
#pragma once

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

// AKM: A stored K x M, staged as [k][m] rows; BKN: B stored K x N, staged as [k][n] rows; TILE: 256 or 128;
// PF: prefetch distance in K tiles (PF + 1 stages of A, PF of B)
#define TILED_MF16(NAME, DT, AKM, BKN, TILE, PF)                                                       \
    {NAME, KIND_TILED, DT, AKM, BKN, 1, TILE, TILE, 64, 256, PF,                                       \
     Cfg16<DT, AKM != 0, BKN != 0, TILE, PF>::LDS_BYTES, 0, &launch_gemm16<Cfg16<DT, AKM != 0, BKN != 0, TILE, PF>>,    \
     BKN, AKM, 0, 0, 1}

// ... with a tile of TM x TN
#define TILED_MF16_MN(NAME, DT, AKM, BKN, TM, TN, PF)                                                  \
    {NAME, KIND_TILED, DT, AKM, BKN, 1, TM, TN, 64, 256, PF,                                           \
     Cfg16<DT, AKM != 0, BKN != 0, TM, PF, TN>::LDS_BYTES, 0,                                          \
     &launch_gemm16<Cfg16<DT, AKM != 0, BKN != 0, TM, PF, TN>>, BKN, AKM, 0, 0, 1}

// ... with BK k per stage
#define TILED_MF16_K(NAME, DT, AKM, BKN, TM, TN, PF, BK)                                               \
    {NAME, KIND_TILED, DT, AKM, BKN, 1, TM, TN, BK, 256, PF,                                           \
     Cfg16<DT, AKM != 0, BKN != 0, TM, PF, TN, BK>::LDS_BYTES, 0,                                      \
     &launch_gemm16<Cfg16<DT, AKM != 0, BKN != 0, TM, PF, TN, BK>>, BKN, AKM, 0, 0, 1}

}  // namespace peak
