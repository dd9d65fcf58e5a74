/*
 * nimbus_calib.h: calibration launches used by the benchmark, exported by the same shared
 * library as nimbus_cop.h.  They measure what the chip sustains on the resources the
 * kernels are bounded by (matrix cores and memory reads for the COP kernel, 64-bit integer
 * arithmetic for the server-side transforms), so that their times can be set against
 * measured ceilings as well as against the published peaks.  Not part of the COP path; for
 * callers that benchmark.
 *
 * Each only enqueues one kernel on `stream` (a hipStream_t, NULL = default) and return at
 * once; the caller times them.  Pointers are DEVICE pointers owned by the caller.
 * Return value: the amount of work enqueued, or -1 for invalid arguments / a refused launch.
 */
#ifndef NIMBUS_CALIB_H
#define NIMBUS_CALIB_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Register-only loop of the int8 matrix-core instruction the COP kernel uses (3 share
 * planes x 7 ciphertext planes into 9 accumulators per wave, Section 3.2's scalar-times-
 * polynomial products after the byte split), `workgroups` workgroups of four waves, `iters`
 * rounds of 21 instructions per wave; operand bytes all zero (random_operands = 0) or
 * pseudo-random (1).  sink: at least workgroups * 1024 bytes, written once.
 * Returns the number of int8 operations (2 per multiply-accumulate) enqueued.
 */
long long nimbus_calib_mfma_i8(int workgroups, int iters, int random_operands, void *sink,
                               size_t sink_bytes, void *stream);

/*
 * Streaming read of `bytes` bytes at `src` (16-byte aligned) with 16-byte loads.
 * sink: at least 4 bytes.  Returns the number of bytes read.
 */
long long nimbus_calib_stream_read(const void *src, size_t bytes, void *sink, void *stream);

/*
 * Register-only loop of the transform butterfly of the server side (Algorithm 1 steps 1
 * and 5 multiply polynomials in the number-theoretic-transform domain, Appendix B.1): every
 * thread of `workgroups` workgroups of 256 runs `iters` rounds of 12 butterflies (three
 * stages over eight values) modulo the odd q < 2^62, with no memory access in the loop.
 * The butterfly is the one the transform kernels run for this modulus: without conditional
 * subtractions and with the shorter quotient estimate for 2^34 <= q < 2^58, the lazy
 * butterfly with one conditional subtraction otherwise.  sink: at least workgroups * 2048
 * bytes, written once.
 * Returns the number of butterflies enqueued.
 */
long long nimbus_calib_butterflies(int workgroups, int iters, unsigned long long q, void *sink,
                                   size_t sink_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* NIMBUS_CALIB_H */
