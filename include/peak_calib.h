/*
 * peak_calib.h - measurement support of the MI355X GEMM library (C ABI).
 *
 * The paper rates a kernel against what the device can do: Section 4.3 gives
 * the devices' documented peaks and Section 6 (Table 1) reports the fraction of
 * the vendor library reached.  A data-sheet peak assumes the data-sheet clock;
 * under a matrix-core load with random operands the chip is power limited and
 * runs slower.  These calls measure, in the caller's process and clock
 * state, what the device sustains when nothing but the matrix cores (or nothing
 * but memory reads) is busy, so that a GEMM time can be quoted against both
 * the published peak and the rate the box can actually issue.  They are used by
 * bench.py only; the GEMM entry points do not depend on them.
 *
 * All pointers named *_dev are DEVICE pointers; the calls enqueue one kernel on
 * `hip_stream` (a hipStream_t passed as void*, NULL = default stream) and
 * return without waiting.  They allocate nothing.  Time them with HIP events.
 */
#ifndef PEAK_CALIB_H
#define PEAK_CALIB_H

#include "peak_gemm.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * MFMA-only loop: one workgroup of 8 waves per compute unit, each wave issuing
 * `iters` x 8 independent 32x32 MFMAs of `dtype` (a peak_dtype_t value: the
 * instruction the GEMM kernels use for it) on register operands, no memory
 * traffic.  random_operands != 0 fills the operand registers with random signs
 * and mantissas (the power draw of a GEMM on random matrices); 0 uses 1.0
 * everywhere (far less switching, higher clock).
 *
 *   out_dev            8-byte aligned, at least 32 bytes, written by the kernel:
 *                      out[0] = shader-clock cycles the loop took on one wave,
 *                      out[1] = ticks of the constant 100 MHz counter over the
 *                      same interval (clock in GHz = 0.1 * out[0] / out[1]).
 *   flops_per_launch   HOST pointer, may be NULL: receives the floating-point
 *                      operations one launch performs on the current device.
 *
 * PEAK_ERR_INVALID_ARG: unknown dtype, iters outside 1..2^24, NULL or misaligned
 * out_dev.  PEAK_ERR_HIP: no device, or the launch failed.
 */
peak_status_t peak_calib_mfma(int32_t dtype, int32_t random_operands, int32_t iters,
                              void *out_dev, void *hip_stream, double *flops_per_launch);

/*
 * Read-only stream: every 16-byte piece of [src_dev, src_dev + bytes) is loaded
 * exactly once (16 bytes per lane, whole cache lines per wave, eight loads in
 * flight per lane, 16 workgroups per compute unit) and nothing is written:
 * bytes / time is the read bandwidth the memory system delivers to a kernel
 * that does nothing else.  Use a buffer well beyond the 256 MB last-level cache.
 *
 *   src_dev  16-byte aligned, `bytes` >= 16 (a trailing piece shorter than 16 bytes is not read)
 *   out_dev  8-byte aligned, at least 32 bytes (written only in a case that does not occur;
 *            it keeps the loads alive)
 */
peak_status_t peak_calib_read(const void *src_dev, size_t bytes, void *out_dev, void *hip_stream);

/*
 * Direct-to-LDS loads only: one workgroup of 4 waves per compute unit, each wave
 * issuing `iters` x 8 loads of 1 KB (buffer_load_dwordx4 ... lds, the staging
 * path of the tiled kernels) from the workgroup's own 64 KB piece of
 * [src_dev, src_dev + bytes), which is served by the L2 after the first pass.
 * bytes_per_workgroup / cycles is what one compute unit's path from the L2
 * into LDS delivers; a 256 x 256 x 64 tile of 16-bit operands needs 64 KB per
 * 2048 cycles of MFMAs, i.e. 32 bytes per cycle of it.
 *
 *   src_dev              16-byte aligned, bytes >= 64 KB x compute units of the device
 *   out_dev              8-byte aligned, 16 bytes per compute unit, written by the kernel:
 *                        out[2 b] = shader-clock cycles workgroup b took,
 *                        out[2 b + 1] = ticks of the constant 100 MHz counter
 *   bytes_per_workgroup  HOST pointer, may be NULL: bytes one workgroup loads per launch
 *   workgroups           HOST pointer, may be NULL: workgroups launched (compute units)
 *
 * PEAK_ERR_INVALID_ARG: NULL or misaligned pointers, iters outside 1..2^20, too
 * few bytes.  PEAK_ERR_HIP: no device, or the launch failed.
 */
peak_status_t peak_calib_lds_load(const void *src_dev, size_t bytes, int32_t iters, void *out_dev, void *hip_stream,
                                  double *bytes_per_workgroup, int32_t *workgroups);

#ifdef __cplusplus
}
#endif
#endif /* PEAK_CALIB_H */
