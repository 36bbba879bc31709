// Test hooks of the library (include/iptq_debug.h): internals exposed so that the tests can
// check them one by one - the integer helpers compiled for the host, the host-side plans and
// layouts, and the two exponential code paths on their own.  Not part of the product API.
#include <hip/hip_runtime.h>

#include "../../include/iptq.h"
#include "../../include/iptq_debug.h"
#include "device_common.h"
#include "kernels.h"
#include "plan.h"
#include "softmax_rows.h"

using namespace iptq;

extern "C" uint32_t iptq_debug_floor_pow2_div(int32_t m_bits, uint32_t sigma)
{
    return floor_pow2_div(m_bits, sigma);
}

extern "C" int iptq_debug_softmax_plan(const iptq_softmax_params_t *p, int64_t rows, int32_t cols,
                                       int32_t has_bias, int64_t bias_period_rows, int64_t *out12)
{
    SoftmaxDev dev;
    int rc = plan_softmax(p, rows, cols, has_bias, bias_period_rows, &dev);
    if (rc != IPTQ_OK || !out12) return rc;
    out12[0] = dev.magic; out12[1] = dev.magic_sh; out12[2] = dev.d_clamp; out12[3] = dev.i0n;
    out12[4] = dev.p_shift; out12[5] = dev.period_magic; out12[6] = dev.period_sh;
    out12[7] = neg_qp_of(dev.d_clamp);
    out12[8] = dev.mode16; out12[9] = dev.mg24; out12[10] = dev.t16;
    out12[11] = dev.pre_rowconst ? (int64_t)dev.pre_dmax : 0;
    return rc;
}

// Layout the run-time-row-length kernels would use for a row length:
// out12 = {slab ok, its lanes per row, its blocks per lane, the same again, wide ok, wide passes, wide slots,
//          1 if the row length has a compiled kernel, 0, workgroup-per-row ok, its wavefronts,
//          its slots}.
extern "C" int iptq_debug_softmax_layout(int32_t cols, int32_t *out12)
{
    if (!out12) return IPTQ_ERR_NULL;
    if (cols < 1 || cols > IPTQ_COLS_MAX) return IPTQ_ERR_SHAPE;
    int a = 0, b = 0;
    out12[0] = rowsdyn_geometry(cols, &a, &b) ? 1 : 0;
    out12[1] = a; out12[2] = b; out12[3] = b;
    a = b = 0;
    out12[4] = wide_geometry(cols, &a, &b) ? 1 : 0;
    out12[5] = a; out12[6] = b;
    a = b = 0;
    out12[7] = softmax_rows_compiled(cols) ? 1 : 0;
    out12[8] = 0;
    a = b = 0;
    out12[9] = wgrow_geometry(cols, &a, &b) ? 1 : 0;
    out12[10] = a; out12[11] = b;
    return IPTQ_OK;
}

// Exponentials of an array of stabilised scores (row maximum 0) through both arithmetic
// paths of the softmax kernels: out32 from the 32-bit lanes, out16 from the packed 16-bit
// lanes (pairs (2i, 2i+1); 0xFFFFFFFF where the plan does not enable that path).  n even.
__global__ void __launch_bounds__(256)
debug_bit_exp_kernel(const int32_t *delta, uint32_t *out32, uint32_t *out16, int64_t n, SoftmaxDev P)
{
    const int64_t i = 2 * ((int64_t)blockIdx.x * 256 + threadIdx.x);
    if (i + 1 >= n + 1 || i >= n) return;
    const int32_t xa = delta[i], xb = delta[i + 1];
    const int32_t lower = -P.d_clamp;
    if (P.variant == 0) {
        out32[i] = bit_exp_dev<0, true>(xa, lower, 0, P);
        out32[i + 1] = bit_exp_dev<0, true>(xb, lower, 0, P);
    } else if (P.variant == 1) {
        out32[i] = bit_exp_dev<1, true>(xa, lower, 0, P);
        out32[i + 1] = bit_exp_dev<1, true>(xb, lower, 0, P);
    } else {
        out32[i] = bit_exp_dev<2, true>(xa, lower, 0, P);
        out32[i + 1] = bit_exp_dev<2, true>(xb, lower, 0, P);
    }
    if (P.mode16 == 0) {
        out16[i] = out16[i + 1] = 0xFFFFFFFFu;
    } else {
        const u16x2 e = P.variant == 0 ? bit_exp_pair<0, true>(xa, xb, 0, P)
                      : P.variant == 1 ? bit_exp_pair<1, true>(xa, xb, 0, P)
                                       : bit_exp_pair<2, true>(xa, xb, 0, P);
        out16[i] = e.x;
        out16[i + 1] = e.y;
    }
}

extern "C" int iptq_debug_bit_exp(const int32_t *d_delta, uint32_t *d_out32, uint32_t *d_out16,
                                  int64_t n, const iptq_softmax_params_t *p, void *stream)
{
    if (!p || !d_delta || !d_out32 || !d_out16) return IPTQ_ERR_NULL;
    if (n < 0 || (n & 1)) return IPTQ_ERR_SHAPE;
    SoftmaxDev dev;
    int rc = plan_softmax(p, 1, 1, 0, 0, &dev);
    if (rc != IPTQ_OK || n == 0) return rc;
    hipLaunchKernelGGL(debug_bit_exp_kernel, dim3((unsigned)((n / 2 + 255) / 256)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), d_delta, d_out32, d_out16, n, dev);
    return hipGetLastError() == hipSuccess ? IPTQ_OK : IPTQ_ERR_HIP;
}
