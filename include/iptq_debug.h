/*
 * iptq_debug.h - test hooks of libiptq.so.  They expose internals (integer helpers, host-side
 * plans and layouts, the two exponential code paths) so that the test-suite can check each on
 * its own; they are not part of the product API (include/iptq.h) and may change with the
 * kernels.  Conventions as in iptq.h: d_* are device pointers, everything else is host memory,
 * return value IPTQ_OK or a negative IPTQ_ERR_* code.
 */
#ifndef IPTQ_DEBUG_H
#define IPTQ_DEBUG_H

#include <stdint.h>

#include "iptq.h"

#ifdef __cplusplus
extern "C" {
#endif

/* floor(2^m_bits / sigma) as the kernels compute it (Newton iteration on integers, Eq. 15),
 * compiled for the host.  1 <= m_bits <= 31; sigma == 0 returns 0. */
uint32_t iptq_debug_floor_pow2_div(int32_t m_bits, uint32_t sigma);

/* The constants the host derives for one softmax launch.  out12 (12 values, may be NULL):
 * {divider multiplier, its shift, clamp D, i0 << N, p shift, period multiplier, its shift,
 *  n(D), packed-16-bit mode, its 24-bit multiplier, its pre-shift,
 *  the clamp of the raw score difference when the requantization in front is folded into Eq. 6
 *  (0: it is not)}. */
int iptq_debug_softmax_plan(const iptq_softmax_params_t *p, int64_t rows, int32_t cols,
                            int32_t has_bias, int64_t bias_period_rows, int64_t *out12);

/* Layouts the run-time-row-length kernels would use for a row length.  out12 (12 values):
 * {slab kernel serves it, its lanes per row, its blocks per lane, the same again,
 *  wavefront-per-row kernel serves it, its passes, its slots, row length has a compiled kernel,
 *  0, workgroup-per-row kernel serves it, its wavefronts, its slots}. */
int iptq_debug_softmax_layout(int32_t cols, int32_t *out12);

/* Exponentials (Eq. 7-14) of n stabilised scores (row maximum 0; n even) through both arithmetic
 * paths of the softmax kernels: d_out32 from the 32-bit lanes, d_out16 from the packed 16-bit
 * lanes (0xFFFFFFFF where the parameters do not enable that path).  All three device arrays
 * hold n elements. */
int iptq_debug_bit_exp(const int32_t *d_delta, uint32_t *d_out32, uint32_t *d_out16, int64_t n,
                       const iptq_softmax_params_t *p, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* IPTQ_DEBUG_H */
