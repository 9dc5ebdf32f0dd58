/*
 * libsparq_probe -- machine ceilings measured on the device the benchmark runs on.
 *
 * Not part of the method: two micro-benchmarks whose results the benchmark prints
 * next to the published peaks, so that a roofline fraction can be read against
 * what this very GPU sustains.
 *   - a loop of nothing but v_mfma_i32_32x32x32_i8 on register operands (the
 *     instruction the contraction of Eq. 1 runs on), with all-zero or random
 *     operand bytes: the matrix pipeline's rate turns out to depend on the data
 *     (the chip lowers its clock under the power the multipliers draw);
 *   - a streaming copy (128-bit loads and stores, grid-stride), the reference for
 *     the HBM-bound trim and dequantisation kernels and the calibration kernel
 *     for the FETCH_SIZE / WRITE_SIZE counters.
 * All pointers are DEVICE pointers owned by the caller; stream is a hipStream_t
 * passed as void*; calls only enqueue work.  Return value: 0 on success, 1 for
 * invalid arguments, 4 if the launch failed (the codes of sparq_status).
 */
#ifndef SPARQ_PROBE_H
#define SPARQ_PROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Operations (2 per multiply-accumulate) one call of sparq_probe_mfma_i8 performs. */
double sparq_probe_mfma_i8_ops(int32_t iters);

/* `operands`: 12 KiB of operand bytes (8 activation + 4 weight fragments of 256 lanes x 16 bytes),
 * `sink`: 256 KiB receiving one word per lane (keeps the loop alive).  One workgroup of four
 * wavefronts per compute unit, each wavefront iters x 16 matrix instructions on a 128 x 64 tile. */
int sparq_probe_mfma_i8(const void *operands, void *sink, int32_t iters, void *stream);

/* dst[i] = src[i] for `bytes` bytes (a multiple of 16; both 16-byte aligned). */
int sparq_probe_copy(const void *src, void *dst, size_t bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SPARQ_PROBE_H */
