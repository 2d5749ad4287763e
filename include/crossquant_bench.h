/*
 * crossquant_bench.h -- calls of libcrossquant.so that are not part of the method: roofline
 * calibration kernels for a benchmark, and a test hook.  A program that only quantizes needs
 * crossquant.h alone.  Conventions (device pointers, stream, return codes) as in crossquant.h.
 */
#ifndef CROSSQUANT_BENCH_H
#define CROSSQUANT_BENCH_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Roofline calibration, not part of the method: kernels that do nothing but stream, so that a
 * benchmark can state what this device sustains next to the published peaks: a plain
 * 16-byte-per-lane read, a copy, and an MFMA-only loop.
 * crossquant_calib_read: reads `bytes` (multiple of 16, src 16-byte aligned); sink (nullable,
 *   device, 8-byte aligned) is only there to keep the loads alive and is normally left untouched.
 * crossquant_calib_copy: dst[0..bytes) = src[0..bytes), both 16-byte aligned, non-overlapping.
 * crossquant_calib_mfma_i8: every SIMD issues iters * 16 independent v_mfma_i32_32x32x32_i8 on
 *   operands held in registers; data_mode 0 = all-zero operands, 1 = bell-shaped int8 codes.
 *   data_mode 3 = the bell-shaped codes on v_mfma_i32_16x16x64_i8, the instruction the linear kernel uses
 *   (iters * 32 instructions per wave, two waves per SIMD).  data_mode 2 = the same, with the operands re-read from LDS every step
 *   the way the linear kernel's inner loop reads them (two waves per SIMD, 8 + 4 fragment reads per 32
 *   instructions = 0.75 KiB per 32 x 32 x 32 worth of multiply-adds; iters * 32 instructions per wave): the ceiling
 *   of a kernel with that wave tile, which no global load, barrier or epilogue burdens.
 *   *ops (HOST pointer, nullable) receives the number of integer operations of the launch.
 * crossquant_calib_mfma_f6: the loop fed from LDS for the A4W4 kernel: v_mfma_f32_16x16x128_f8f6f4 on FP6 operands
 *   holding bell-shaped INT4-like codes, 8 + 4 tiles (a 16-byte and an 8-byte read per lane each) per 32 instructions,
 *   two waves per SIMD, iters * 32 instructions per wave.  *ops as above (2 per multiply-add).
 */
int crossquant_calib_read(const void *src, int64_t bytes, unsigned long long *sink, void *stream);
int crossquant_calib_copy(const void *src, void *dst, int64_t bytes, void *stream);
int crossquant_calib_mfma_i8(int iters, int data_mode, int *sink, double *ops, void *stream);
int crossquant_calib_mfma_f6(int iters, int *sink, double *ops, void *stream);

/*
 * Test hook for crossquant_absmax_quantize_single_read: the number of polls a block makes at the grid
 * barrier before it gives up (default 2^22, seconds).  0 makes every block give up at once, so the failure
 * path (NaN in row_scale / col_scale, codes not written) can be exercised without a GPU ever
 * waiting.  Process-wide, not thread-safe; pass 1u << 22 to restore the default.
 */
void crossquant_debug_set_barrier_polls(unsigned polls);

#ifdef __cplusplus
}
#endif
#endif /* CROSSQUANT_BENCH_H */
