// C ABI of the library: argument checks (host only), then one or two kernel launches on
// the caller's stream.  Declarations and contracts: include/iptq.h.
#include <hip/hip_runtime.h>

#include "../../include/iptq.h"
#include "device_common.h"
#include "kernels.h"
#include "plan.h"
#include "softmax_rows.h"

using namespace iptq;

static int hip_rc(hipError_t e) { return e == hipSuccess ? IPTQ_OK : IPTQ_ERR_HIP; }

static bool overlap(const void *a, int64_t na, const void *b, int64_t nb)
{
    const uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
    return a0 < b0 + (uintptr_t)nb && b0 < a0 + (uintptr_t)na;
}

extern "C" int iptq_requant(const int32_t *d_in, void *d_out, int64_t n, int32_t out_is_signed,
                            const iptq_dyadic_t *p, void *stream)
{
    if (!p) return IPTQ_ERR_NULL;
    if (n < 0) return IPTQ_ERR_SHAPE;
    DyadicDev dev;
    int rc = plan_requant(p, out_is_signed, &dev);
    if (rc != IPTQ_OK) return rc;
    if (n == 0) return IPTQ_OK;
    if (!d_in || !d_out) return IPTQ_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(d_in) & 3) return IPTQ_ERR_ALIGN;
    if (overlap(d_in, n * 4, d_out, n)) return IPTQ_ERR_PARAM;
    return hip_rc(requant_dispatch(d_in, d_out, n, dev, static_cast<hipStream_t>(stream)));
}

// Validates one softmax problem and fills its launch record.  rows == 0 is valid.
static int softmax_call(const int32_t *d_scores, const int32_t *d_bias, int64_t bias_period_rows,
                        void *d_out, int64_t rows, int32_t cols, const iptq_softmax_params_t *p,
                        SoftmaxCall *out)
{
    if (!p) return IPTQ_ERR_NULL;
    int rc = plan_softmax(p, rows, cols, d_bias != nullptr, bias_period_rows, &out->P);
    if (rc != IPTQ_OK) return rc;
    out->scores = d_scores; out->bias = d_bias; out->out = static_cast<uint8_t *>(d_out);
    out->rows = rows; out->out_bits = p->out_bits; out->algo = p->algo;
    if (rows == 0) return IPTQ_OK;
    if (!d_scores || !d_out) return IPTQ_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(d_scores) & 3) || (reinterpret_cast<uintptr_t>(d_bias) & 3))
        return IPTQ_ERR_ALIGN;
    if (overlap(d_scores, rows * cols * 4, d_out, rows * cols)) return IPTQ_ERR_PARAM;
    return IPTQ_OK;
}

static int gelu_call(const int8_t *d_in, int8_t *d_out, int64_t n, const iptq_gelu_params_t *p,
                     GeluCall *out)
{
    if (!p) return IPTQ_ERR_NULL;
    if (n < 0) return IPTQ_ERR_SHAPE;
    int rc = plan_gelu(p, 1, &out->P);
    if (rc != IPTQ_OK) return rc;
    out->in = d_in; out->out = d_out; out->n = n; out->force_direct = p->algo == IPTQ_ALGO_GENERIC;
    if (n == 0) return IPTQ_OK;
    if (!d_in || !d_out) return IPTQ_ERR_NULL;
    if (d_in != d_out && overlap(d_in, n, d_out, n)) return IPTQ_ERR_PARAM;
    return IPTQ_OK;
}

extern "C" int iptq_softmax_i32(const int32_t *d_scores, const int32_t *d_bias,
                                int64_t bias_period_rows, void *d_out, int64_t rows, int32_t cols,
                                const iptq_softmax_params_t *p, void *stream)
{
    SoftmaxCall call;
    int rc = softmax_call(d_scores, d_bias, bias_period_rows, d_out, rows, cols, p, &call);
    if (rc != IPTQ_OK || rows == 0) return rc;
    return hip_rc(softmax_dispatch(&call, 1, cols, static_cast<hipStream_t>(stream)));
}

extern "C" int iptq_softmax_i32_batch(const iptq_softmax_problem_t *problems, int32_t n_problems,
                                      int32_t cols, void *stream)
{
    if (n_problems < 0) return IPTQ_ERR_SHAPE;
    if (n_problems == 0) return IPTQ_OK;
    if (!problems) return IPTQ_ERR_NULL;
    if (n_problems > IPTQ_BATCH_MAX) return IPTQ_ERR_SHAPE;
    SoftmaxCall calls[IPTQ_BATCH_MAX];
    int n = 0;
    for (int32_t i = 0; i < n_problems; ++i) {           // every problem is checked before any launch
        const iptq_softmax_problem_t &q = problems[i];
        int rc = softmax_call(q.d_scores, q.d_bias, q.bias_period_rows, q.d_out, q.rows, cols,
                              &q.params, &calls[n]);
        if (rc != IPTQ_OK) return rc;
        if (q.rows > 0) ++n;
    }
    if (n == 0) return IPTQ_OK;
    return hip_rc(softmax_dispatch(calls, n, cols, static_cast<hipStream_t>(stream)));
}

extern "C" int iptq_gelu_i8(const int8_t *d_in, int8_t *d_out, int64_t n,
                            const iptq_gelu_params_t *p, void *stream)
{
    GeluCall call;
    int rc = gelu_call(d_in, d_out, n, p, &call);
    if (rc != IPTQ_OK || n == 0) return rc;
    return hip_rc(gelu_i8_dispatch(&call, 1, static_cast<hipStream_t>(stream)));
}

extern "C" int iptq_gelu_i8_batch(const iptq_gelu_problem_t *problems, int32_t n_problems,
                                  void *stream)
{
    if (n_problems < 0) return IPTQ_ERR_SHAPE;
    if (n_problems == 0) return IPTQ_OK;
    if (!problems) return IPTQ_ERR_NULL;
    if (n_problems > IPTQ_BATCH_MAX) return IPTQ_ERR_SHAPE;
    GeluCall calls[IPTQ_BATCH_MAX];
    int n = 0;
    for (int32_t i = 0; i < n_problems; ++i) {
        const iptq_gelu_problem_t &q = problems[i];
        int rc = gelu_call(q.d_in, q.d_out, q.n, &q.params, &calls[n]);
        if (rc != IPTQ_OK) return rc;
        if (q.n > 0) ++n;
    }
    if (n == 0) return IPTQ_OK;
    return hip_rc(gelu_i8_dispatch(calls, n, static_cast<hipStream_t>(stream)));
}

extern "C" int iptq_gelu_i32(const int32_t *d_in, int8_t *d_out, int64_t n,
                             const iptq_gelu_params_t *p, void *stream)
{
    if (!p) return IPTQ_ERR_NULL;
    if (n < 0) return IPTQ_ERR_SHAPE;
    GeluDev dev;
    int rc = plan_gelu(p, 0, &dev);
    if (rc != IPTQ_OK) return rc;
    if (n == 0) return IPTQ_OK;
    if (!d_in || !d_out) return IPTQ_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(d_in) & 3) return IPTQ_ERR_ALIGN;
    if (overlap(d_in, n * 4, d_out, n)) return IPTQ_ERR_PARAM;
    return hip_rc(gelu_i32_dispatch(d_in, d_out, n, dev, p->algo == IPTQ_ALGO_GENERIC, static_cast<hipStream_t>(stream)));
}

extern "C" int iptq_softmax_i32_layers(const int32_t *d_scores, int64_t in_stride, void *d_out,
                                       int64_t out_stride, int64_t rows, int32_t cols,
                                       int32_t n_layers, const iptq_softmax_params_t *p,
                                       void *stream)
{
    if (n_layers < 0 || in_stride < 0 || out_stride < 0) return IPTQ_ERR_SHAPE;
    if (n_layers == 0) return IPTQ_OK;
    if (!p) return IPTQ_ERR_NULL;
    if (n_layers > 1 && rows > 0 && (in_stride < rows * cols || out_stride < rows * cols))
        return IPTQ_ERR_SHAPE;
    // every layer is checked before the first launch
    for (int32_t l = 0; l < n_layers; ++l) {
        SoftmaxCall call;
        int rc = softmax_call(d_scores ? d_scores + l * in_stride : nullptr, nullptr, 0,
                              d_out ? static_cast<uint8_t *>(d_out) + l * out_stride : nullptr, rows,
                              cols, &p[l], &call);
        if (rc != IPTQ_OK) return rc;
    }
    if (rows == 0) return IPTQ_OK;
    for (int32_t base = 0; base < n_layers; base += IPTQ_BATCH_MAX) {
        SoftmaxCall calls[IPTQ_BATCH_MAX];
        const int32_t cnt = n_layers - base < IPTQ_BATCH_MAX ? n_layers - base : IPTQ_BATCH_MAX;
        for (int32_t i = 0; i < cnt; ++i) {
            const int32_t l = base + i;
            softmax_call(d_scores + l * in_stride, nullptr, 0, static_cast<uint8_t *>(d_out) + l * out_stride,
                         rows, cols, &p[l], &calls[i]);
        }
        int rc = hip_rc(softmax_dispatch(calls, cnt, cols, static_cast<hipStream_t>(stream)));
        if (rc != IPTQ_OK) return rc;
    }
    return IPTQ_OK;
}

extern "C" int iptq_gelu_i8_layers(const int8_t *d_in, int64_t in_stride, int8_t *d_out,
                                   int64_t out_stride, int64_t n, int32_t n_layers,
                                   const iptq_gelu_params_t *p, void *stream)
{
    if (n_layers < 0 || in_stride < 0 || out_stride < 0 || n < 0) return IPTQ_ERR_SHAPE;
    if (n_layers == 0) return IPTQ_OK;
    if (!p) return IPTQ_ERR_NULL;
    if (n_layers > 1 && (in_stride < n || out_stride < n)) return IPTQ_ERR_SHAPE;
    for (int32_t l = 0; l < n_layers; ++l) {
        GeluCall call;
        int rc = gelu_call(d_in ? d_in + l * in_stride : nullptr, d_out ? d_out + l * out_stride : nullptr,
                           n, &p[l], &call);
        if (rc != IPTQ_OK) return rc;
    }
    if (n == 0) return IPTQ_OK;
    for (int32_t base = 0; base < n_layers; base += IPTQ_BATCH_MAX) {
        GeluCall calls[IPTQ_BATCH_MAX];
        const int32_t cnt = n_layers - base < IPTQ_BATCH_MAX ? n_layers - base : IPTQ_BATCH_MAX;
        for (int32_t i = 0; i < cnt; ++i) {
            const int32_t l = base + i;
            gelu_call(d_in + l * in_stride, d_out + l * out_stride, n, &p[l], &calls[i]);
        }
        int rc = hip_rc(gelu_i8_dispatch(calls, cnt, static_cast<hipStream_t>(stream)));
        if (rc != IPTQ_OK) return rc;
    }
    return IPTQ_OK;
}

// ---- host-side test hooks (not part of the public header): the same source the kernels
// run, compiled for the host, so that integer helpers can be checked exhaustively without
// a GPU.
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
    out12[8] = dev.mode16; out12[9] = dev.mg24; out12[10] = dev.t16; out12[11] = 0;
    return rc;
}

// Layout the run-time-row-length kernels would use for a row length:
// out12 = {slab ok, its lanes per row, its blocks per lane, the same again, wide ok, wide passes, wide slots,
//          1 if the row length has a compiled kernel, 0, workgroup-per-row ok, its wavefronts,
//          its slots}.
extern "C" int iptq_debug_softmax_layout(int32_t cols, int32_t *out9)
{
    if (!out9) return IPTQ_ERR_NULL;
    if (cols < 1 || cols > IPTQ_COLS_MAX) return IPTQ_ERR_SHAPE;
    int a = 0, b = 0;
    out9[0] = rowsdyn_geometry(cols, &a, &b) ? 1 : 0;
    out9[1] = a; out9[2] = b; out9[3] = b;
    a = b = 0;
    out9[4] = wide_geometry(cols, &a, &b) ? 1 : 0;
    out9[5] = a; out9[6] = b;
    a = b = 0;
    out9[7] = softmax_rows_compiled(cols) ? 1 : 0;
    out9[8] = 0;
    a = b = 0;
    out9[9] = wgrow_geometry(cols, &a, &b) ? 1 : 0;
    out9[10] = a; out9[11] = b;
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
    } else {
        out32[i] = bit_exp_dev<1, true>(xa, lower, 0, P);
        out32[i + 1] = bit_exp_dev<1, true>(xb, lower, 0, P);
    }
    if (P.mode16 == 0) {
        out16[i] = out16[i + 1] = 0xFFFFFFFFu;
    } else {
        const u16x2 e = P.variant == 0 ? bit_exp_pair<0, true>(xa, xb, 0, P) : bit_exp_pair<1, true>(xa, xb, 0, P);
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
    return hip_rc(hipGetLastError());
}
