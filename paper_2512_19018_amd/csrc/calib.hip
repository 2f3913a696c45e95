// Measurement support for the bench: what the device sustains with nothing but
// the matrix cores busy, with nothing but reads from memory, and with nothing but
// direct-to-LDS loads from the L2, measured in the same process and clock state
// as the GEMM runs they are compared with.
#include "../../include/peak_calib.h"

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int CALIB_WAVES = 8;        // per workgroup: two per SIMD
constexpr int CALIB_ACCS = 8;         // independent accumulators per wave: no MFMA waits on the one before

__device__ __forceinline__ uint32_t lcg(uint32_t &h)
{
    h = h * 1664525u + 1013904223u;
    return h >> 8;
}

// Operands like those of a GEMM on random matrices: random sign and mantissa,
// exponents within a few binades of 1.  (Constant operands toggle far fewer
// wires in the multipliers and let the chip hold a much higher clock.)
template <int DT>
__device__ __forceinline__ u32x4 operand(uint32_t &h, bool random)
{
    u32x4 v;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        if (DT == 0) {                 // fp32
            const uint32_t r = lcg(h);
            v[e] = random ? ((r & 0x807FFFFFu) | ((((r >> 24) & 3) + 0x7D) << 23)) : 0x3F800000u;
        } else if (DT == 2) {          // bf16: 1 sign, 8 exponent, 7 mantissa bits
            uint32_t lo = lcg(h) & 0xFFFF, hi = lcg(h) & 0xFFFF;
            lo = (lo & 0x807F) | ((((lo >> 8) & 3) + 0x7D) << 7);
            hi = (hi & 0x807F) | ((((hi >> 8) & 3) + 0x7D) << 7);
            v[e] = random ? (lo | (hi << 16)) : 0x3F803F80u;
        } else {                       // f16: 1 sign, 5 exponent, 10 mantissa bits
            uint32_t lo = lcg(h) & 0xFFFF, hi = lcg(h) & 0xFFFF;
            lo = (lo & 0x83FF) | ((((lo >> 11) & 3) + 0x0D) << 10);
            hi = (hi & 0x83FF) | ((((hi >> 11) & 3) + 0x0D) << 10);
            v[e] = random ? (lo | (hi << 16)) : 0x3C003C00u;
        }
    }
    return v;
}

template <int DT>
__global__ __launch_bounds__(CALIB_WAVES * 64) void mfma_only_kernel(uint64_t *out, int iters, int random)
{
    uint32_t h = (threadIdx.x * 2654435761u) ^ (blockIdx.x * 40503u) ^ 0x9E3779B9u;
    u32x4 a[4], b[2];
#pragma unroll
    for (int i = 0; i < 4; ++i) a[i] = operand<DT>(h, random != 0);
#pragma unroll
    for (int i = 0; i < 2; ++i) b[i] = operand<DT>(h, random != 0);
    f32x16 acc[CALIB_ACCS];
#pragma unroll
    for (int i = 0; i < CALIB_ACCS; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.0f;

    const long long c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < CALIB_ACCS; ++i) {
            if (DT == 2)
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[i & 3]),
                                                                 __builtin_bit_cast(bf16x8, b[i >> 2]), acc[i], 0, 0, 0);
            else if (DT == 1)
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a[i & 3]),
                                                                __builtin_bit_cast(f16x8, b[i >> 2]), acc[i], 0, 0, 0);
            else
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(__builtin_bit_cast(float, a[i & 3][0]),
                                                              __builtin_bit_cast(float, b[i >> 2][0]), acc[i], 0, 0, 0);
        }
    }
    const long long c1 = clock64(), w1 = wall_clock64();
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < CALIB_ACCS; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[i][v];
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        out[0] = (uint64_t)(c1 - c0);              // shader clock cycles of the loop
        out[1] = (uint64_t)(w1 - w0);              // ticks of the constant 100 MHz counter
    }
    if (s == 12345.678f) out[2] = (uint64_t)s;     // keeps the loop alive; practically never taken
}

// Every 16-byte piece of [src, src + bytes) is read once, 16 bytes per lane,
// consecutive lanes on consecutive pieces, eight loads in flight per lane.
__global__ __launch_bounds__(256) void read_only_kernel(const u32x4 *src, uint64_t nvec, uint64_t *out)
{
    constexpr int U = 8;
    const uint64_t per_block = (nvec + gridDim.x - 1) / gridDim.x;
    const uint64_t begin = per_block * blockIdx.x;
    uint64_t end = begin + per_block;
    if (end > nvec) end = nvec;
    u32x4 x = {0u, 0u, 0u, 0u};
    uint64_t i = begin + threadIdx.x;
    for (; i + (uint64_t)(U - 1) * 256 < end; i += (uint64_t)U * 256) {
        u32x4 t[U];
#pragma unroll
        for (int u = 0; u < U; ++u) t[u] = __builtin_nontemporal_load(src + i + (uint64_t)u * 256);
#pragma unroll
        for (int u = 0; u < U; ++u) x ^= t[u];
    }
    for (; i < end; i += 256) x ^= __builtin_nontemporal_load(src + i);
    if ((x[0] ^ x[1] ^ x[2] ^ x[3]) == 0x9E3779B9u && x[0] == 0x12345678u) out[3] = x[1];   // practically never taken
}

// Direct-to-LDS loads and nothing else: each wave of a 4-wave workgroup (one workgroup per compute unit) issues
// `iters` x 8 loads of 1 KB (16 bytes per lane) from its workgroup's own 64 KB piece of the source, which stays
// in the L2 after the first pass, into a ring in LDS.  out[2 b], out[2 b + 1] = shader-clock cycles workgroup b
// took, and the constant 100 MHz counter's ticks.
constexpr int LDSLOAD_REGION = 64 * 1024;
__global__ __launch_bounds__(256) void lds_load_kernel(const char *src, uint64_t *out, int iters)
{
    __shared__ __attribute__((aligned(1024))) char ring[128 * 1024];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const char *base = src + (size_t)blockIdx.x * LDSLOAD_REGION;
    __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc((void *)base, 0, LDSLOAD_REGION, 0x00020000);
    const long long c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int chunk = ((it * 8 + i) * 4 + wave) & 0xFFFF;          // 1 KB piece
            const int off = (chunk * 1024) % LDSLOAD_REGION + lane * 16;     // inside the descriptor's 64 KB
            __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (__attribute__((address_space(3))) void *)(ring + (chunk % 128) * 1024), 16, off, 0, 0, 0);
        }
        if ((it & 3) == 3) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    const long long c1 = clock64(), w1 = wall_clock64();
    __syncthreads();
    if (threadIdx.x == 0) {
        out[2 * blockIdx.x] = (uint64_t)(c1 - c0);
        out[2 * blockIdx.x + 1] = (uint64_t)(w1 - w0);
    }
    if (ring[threadIdx.x] == 0x5A && ring[threadIdx.x + 256] == 0x3C && iters < 0) out[0] = 0;   // keeps the ring alive; never taken
}

}  // namespace

extern "C" {

peak_status_t peak_calib_mfma(int32_t dtype, int32_t random_operands, int32_t iters, void *out_dev, void *hip_stream,
                              double *flops_per_launch)
{
    if (!out_dev || (uintptr_t)out_dev % 8 || iters < 1 || iters > (1 << 24)) return PEAK_ERR_INVALID_ARG;
    if (dtype != PEAK_DT_F32 && dtype != PEAK_DT_F16 && dtype != PEAK_DT_BF16) return PEAK_ERR_INVALID_ARG;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
        return PEAK_ERR_HIP;
    const dim3 grid((unsigned)cus), block(CALIB_WAVES * 64);
    hipStream_t s = (hipStream_t)hip_stream;
    uint64_t *out = (uint64_t *)out_dev;
    if (dtype == PEAK_DT_BF16) hipLaunchKernelGGL(mfma_only_kernel<2>, grid, block, 0, s, out, iters, random_operands);
    else if (dtype == PEAK_DT_F16) hipLaunchKernelGGL(mfma_only_kernel<1>, grid, block, 0, s, out, iters, random_operands);
    else hipLaunchKernelGGL(mfma_only_kernel<0>, grid, block, 0, s, out, iters, random_operands);
    if (hipGetLastError() != hipSuccess) return PEAK_ERR_HIP;
    if (flops_per_launch) {
        const double per_mfma = dtype == PEAK_DT_F32 ? 2.0 * 32 * 32 * 2 : 2.0 * 32 * 32 * 16;
        *flops_per_launch = per_mfma * CALIB_ACCS * (double)iters * CALIB_WAVES * (double)cus;
    }
    return PEAK_OK;
}

peak_status_t peak_calib_read(const void *src_dev, size_t bytes, void *out_dev, void *hip_stream)
{
    if (!src_dev || !out_dev || (uintptr_t)src_dev % 16 || (uintptr_t)out_dev % 8 || bytes < 16) return PEAK_ERR_INVALID_ARG;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
        return PEAK_ERR_HIP;
    hipLaunchKernelGGL(read_only_kernel, dim3((unsigned)cus * 16), dim3(256), 0, (hipStream_t)hip_stream,
                       (const u32x4 *)src_dev, (uint64_t)(bytes / 16), (uint64_t *)out_dev);
    return hipGetLastError() == hipSuccess ? PEAK_OK : PEAK_ERR_HIP;
}

peak_status_t peak_calib_lds_load(const void *src_dev, size_t bytes, int32_t iters, void *out_dev, void *hip_stream,
                                  double *bytes_per_workgroup, int32_t *workgroups)
{
    if (!src_dev || !out_dev || (uintptr_t)src_dev % 16 || (uintptr_t)out_dev % 8 || iters < 1 || iters > (1 << 20)) return PEAK_ERR_INVALID_ARG;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
        return PEAK_ERR_HIP;
    if (bytes < (size_t)cus * LDSLOAD_REGION) return PEAK_ERR_INVALID_ARG;
    hipLaunchKernelGGL(lds_load_kernel, dim3((unsigned)cus), dim3(256), 0, (hipStream_t)hip_stream,
                       (const char *)src_dev, (uint64_t *)out_dev, iters);
    if (hipGetLastError() != hipSuccess) return PEAK_ERR_HIP;
    if (bytes_per_workgroup) *bytes_per_workgroup = (double)iters * 8.0 * 4.0 * 1024.0;
    if (workgroups) *workgroups = cus;
    return PEAK_OK;
}

}  // extern "C"
