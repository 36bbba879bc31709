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
                        SoftmaxCall *out, const int32_t *d_mask = nullptr, int64_t n_windows = 0,
                        int64_t heads = 0, const uint64_t *d_mask_bits = nullptr)
{
    if (!p) return IPTQ_ERR_NULL;
    int rc = plan_softmax(p, rows, cols, d_bias != nullptr, bias_period_rows, &out->P);
    if (rc != IPTQ_OK) return rc;
    if (d_mask && d_mask_bits) return IPTQ_ERR_PARAM;     // one form of the mask or the other
    if (d_mask || d_mask_bits) {
        rc = plan_softmax_mask(n_windows, heads, cols, &out->P);
        if (rc != IPTQ_OK) return rc;
        if ((reinterpret_cast<uintptr_t>(d_mask) & 3) || (reinterpret_cast<uintptr_t>(d_mask_bits) & 7))
            return IPTQ_ERR_ALIGN;
    }
    out->mask = d_mask;
    out->mask_bits = d_mask_bits;
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

extern "C" int iptq_softmax_i32_windowed(const int32_t *d_scores, const int32_t *d_bias,
                                         int64_t bias_period_rows, const int32_t *d_mask,
                                         int32_t n_windows, int32_t heads, void *d_out, int64_t rows,
                                         int32_t cols, const iptq_softmax_params_t *p, void *stream)
{
    SoftmaxCall call;
    int rc = softmax_call(d_scores, d_bias, bias_period_rows, d_out, rows, cols, p, &call, d_mask,
                          n_windows, heads);
    if (rc != IPTQ_OK || rows == 0) return rc;
    return hip_rc(softmax_dispatch(&call, 1, cols, static_cast<hipStream_t>(stream)));
}

extern "C" int iptq_softmax_i32_windowed_bits(const int32_t *d_scores, const int32_t *d_bias,
                                              int64_t bias_period_rows, const uint64_t *d_mask_bits,
                                              int32_t n_windows, int32_t heads, void *d_out,
                                              int64_t rows, int32_t cols,
                                              const iptq_softmax_params_t *p, void *stream)
{
    SoftmaxCall call;
    int rc = softmax_call(d_scores, d_bias, bias_period_rows, d_out, rows, cols, p, &call, nullptr,
                          n_windows, heads, d_mask_bits);
    if (rc != IPTQ_OK || rows == 0) return rc;
    return hip_rc(softmax_dispatch(&call, 1, cols, static_cast<hipStream_t>(stream)));
}

extern "C" int iptq_pack_window_mask(const int32_t *d_mask, int32_t n_windows, int32_t cols,
                                     uint64_t *d_mask_bits, void *stream)
{
    if (n_windows < 0 || cols < 1 || cols > IPTQ_COLS_MAX) return IPTQ_ERR_SHAPE;
    if (n_windows == 0) return IPTQ_OK;
    if (!d_mask || !d_mask_bits) return IPTQ_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(d_mask) & 3) || (reinterpret_cast<uintptr_t>(d_mask_bits) & 7))
        return IPTQ_ERR_ALIGN;
    const int64_t n_queries = (int64_t)n_windows * cols;
    if (n_queries * cols >= ((int64_t)1 << 40)) return IPTQ_ERR_SHAPE;
    if (overlap(d_mask, n_queries * cols * 4, d_mask_bits, n_queries * ((cols + 63) / 64) * 8))
        return IPTQ_ERR_PARAM;
    return hip_rc(pack_window_mask_dispatch(d_mask, n_queries, cols, d_mask_bits,
                                            static_cast<hipStream_t>(stream)));
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
                              &q.params, &calls[n], q.d_mask, q.n_windows, q.heads, q.d_mask_bits);
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

extern "C" int iptq_softmax_kernel_family(int32_t cols, int32_t *family, int32_t *lanes,
                                          int32_t *blocks)
{
    if (!family || !lanes || !blocks) return IPTQ_ERR_NULL;
    if (cols < 1 || cols > IPTQ_COLS_MAX) return IPTQ_ERR_SHAPE;
    int a = 0, b = 0;
    *lanes = 0; *blocks = 0;
    if (softmax_rows_compiled(cols)) { *family = IPTQ_FAMILY_COMPILED; return IPTQ_OK; }
    if (rowsdyn_geometry(cols, &a, &b)) { *family = IPTQ_FAMILY_SLAB; *lanes = a; *blocks = b; return IPTQ_OK; }
    if (wide_geometry(cols, &a, &b)) { *family = IPTQ_FAMILY_WAVEFRONT_PER_ROW; *lanes = 64; *blocks = a; return IPTQ_OK; }
    if (wgrow_geometry(cols, &a, &b)) { *family = IPTQ_FAMILY_WORKGROUP_PER_ROW; *lanes = 64 * a; *blocks = b; return IPTQ_OK; }
    *family = IPTQ_FAMILY_THREE_PASS;
    return IPTQ_OK;
}
