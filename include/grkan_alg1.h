/*
 * grkan_alg1.h - the paper's Algorithm 1 (the original KAT backward pass with
 * one global atomic add per element and coefficient), restated as a
 * MEASUREMENT BASELINE.  It is not part of the product path: grkan_bwd never
 * calls it.  It exists to restate, on MI355X, the two comparisons the FlashKAT
 * paper makes against it (Sec. "Revisiting Speed, Utilization and Stalls",
 * Table 3: run time; Sec. "Reduced Gradient Rounding Error", Table 5 and the
 * appendix: rounding error of dA / dB, which depends on the order in which the
 * atomics land and therefore changes from run to run).
 */
#ifndef GRKAN_ALG1_H_
#define GRKAN_ALG1_H_

#include "grkan.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Algorithm 1, float32: a 1-D grid of ceil(rows*D / 256) blocks of 256
 * threads; each thread takes one element, reads its group's ten coefficients
 * from global memory, computes dx and the ten gradient terms, and adds each
 * term to dA / dB with a global float atomic.
 *
 * x, dy, dx: DEVICE float32 [rows, D]; A [G,6], B [G,4], dA [G,6], dB [G,4]:
 * DEVICE float32.  dA and dB are zeroed on the stream first and then
 * accumulated into, so they are overwritten as in grkan_bwd.  Asynchronous on
 * `hip_stream`.  Same status codes as grkan_bwd; rows * D must be below 2^40.
 */
grkan_status_t grkan_alg1_bwd(const float *x, const float *dy, const float *A, const float *B,
                              float *dx, float *dA, float *dB,
                              int64_t rows, int32_t D, int32_t G, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* GRKAN_ALG1_H_ */
