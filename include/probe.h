/*
 * Measured peaks of the device the library runs on: how fast the matrix pipes go when they
 * do nothing but multiply, and how fast memory is read when it is only streamed.  The
 * nominal figures (2516.6 TFLOP/s bf16, 8 TB/s) assume the nominal clock; under sustained
 * matrix-core load the chip clocks lower, and a kernel's distance from what the hardware
 * actually delivers is the more useful number next to its roofline fraction (the paper's
 * profiler feedback, Sec. 3.3, likewise names the bounding resource and the share of its peak).
 * Measurement helpers only: nothing in the GEMM or rotary paths calls them.
 *
 * Both calls enqueue on `hip_stream` (NULL = default stream), WAIT for the device, create
 * and destroy two HIP events, and allocate nothing.  Status codes are those of gemm.h.
 */
#ifndef MI355GEMM_PROBE_H
#define MI355GEMM_PROBE_H

#include "gemm.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * probe_mfma_peak - every CU runs 8 waves of v_mfma_f32_32x32x16 (dtype GEMM_BF16 or
 * GEMM_F16) or v_mfma_f32_32x32x64_f8f6f4 (GEMM_F8E4M3) on register operands with pseudo-random signs and significands (magnitude about
 * 2^-6), the accumulator footprint of the 256x256 GEMM tile (8 independent 32x32
 * accumulators per wave), no memory traffic.  refresh_operands = 0: the same six operand
 * registers are re-used in rotation (the classic peak loop); 1: their sign and significand
 * bits are flipped by a fresh pseudo-random word before every step, so that the multipliers
 * see new data every time, as in a real product (the chip is power-limited: this runs at a
 * lower clock).  Repeats launches until at least `min_seconds` have been measured.
 * `sink`: DEVICE pointer to at least 4 bytes (written only if an accumulator takes an
 * impossible value; it keeps the loop alive).
 * *tflops receives 2 * multiply-adds / time / 1e12.
 */
int probe_mfma_peak(int dtype, int refresh_operands, void* sink, void* hip_stream, double min_seconds,
                    double* tflops);

/*
 * probe_mfma16_peak - the same loop on v_mfma_f32_16x16x32 (dtype GEMM_BF16 or GEMM_F16), the shape
 * the default 16-bit GEMM kernel multiplies with: 8 waves per CU, the accumulator footprint of a
 * 128x64 wave block (32 independent 16x16 accumulators per wave), 12 operand registers sets.
 * Arguments, blocking behaviour and errors as probe_mfma_peak (GEMM_F8E4M3 is refused).
 */
int probe_mfma16_peak(int dtype, int refresh_operands, void* sink, void* hip_stream, double min_seconds,
                      double* tflops);

/*
 * probe_read_peak - streams `bytes` (a multiple of 16384, at least 1 GiB so that the 256 MB
 * last-level cache cannot serve it) from the DEVICE buffer `src` once per launch with the
 * access pattern of the skinny GEMV (a wave reads 16 KB contiguous with 16 loads of 16 bytes
 * per lane in flight, non-temporal), repeats until `min_seconds` have been measured.
 * *gbytes_per_s receives bytes read / time / 1e9.  `sink` as above.
 */
int probe_read_peak(const void* src, size_t bytes, void* sink, void* hip_stream, double min_seconds,
                    double* gbytes_per_s);

#ifdef __cplusplus
}
#endif
#endif /* MI355GEMM_PROBE_H */
