// Host-only: the Unified Metric that assigns an approximation function to each activation
// layer (Section 4.5, Eq. 16-20).  It runs once, offline, on real-valued calibration
// activations and the dequantized output of each candidate; its result is the `variant` field
// the kernels take.  IEEE double throughout; no HIP calls.
#include <math.h>
#include <stdint.h>

#include "../../include/iptq.h"

namespace {

// integer operations per element of one layer, counted from the steps listed at
// iptq_softmax_params_t / iptq_gelu_params_t (a reduction once per element)
const int kSoftmaxCommonOps = 2     // Eq. 6: compare for the maximum, subtract it
                              + 4   // Eq. 7: two shifts, an add, a subtract
                              + 4   // Eq. 8: negate, divide, multiply and subtract (remainder)
                              + 2   // Eq. 9: shift left by N, right by q
                              + 1   // row sum
                              + 2;  // Eq. 15: multiply by the row's factor, shift
const int kSoftmaxFractionOps[3] = {3,     // Eq. 10: negate, shift, add 1/S
                                    7,     // Eq. 13-14: negate, three shifts, two adds, add 1/S
                                    10};   // second-degree term: square, divide, add on top
const int kSoftmaxRowOps = 1;              // floor(2^M / sum), once per row
const int kGeluOps[2] = {17,   // centre, sign, abs, min, add b, square, add 1, times sign, add 1, shift,
                               // times x, requantization (multiply, add, shift, add zero-point, two clamps)
                         18};  // the quartic reuses the square: one more multiply

// log(1 + exp(x)) (Eq. 17) without overflow: both branches are the same function
double softplus(double x)
{
    if (isinf(x)) return x > 0 ? x : 0.0;
    return x > 0 ? x + log1p(exp(-x)) : log1p(exp(x));
}

}  // namespace

extern "C" int64_t iptq_softmax_op_count(int32_t variant, int64_t rows, int32_t cols)
{
    if (variant < 0 || variant > 2 || rows < 0 || cols < 1) return -1;
    return rows * cols * (int64_t)(kSoftmaxCommonOps + kSoftmaxFractionOps[variant]) + rows * kSoftmaxRowOps;
}

extern "C" int64_t iptq_gelu_op_count(int32_t variant, int64_t n)
{
    if (variant < 0 || variant > 1 || n < 0) return -1;
    return n * (int64_t)kGeluOps[variant];
}

extern "C" int iptq_unified_metric(const double *x, const double *x_hat, int64_t n, double op_count,
                                   int32_t mode, iptq_metric_t *out)
{
    if (!x || !x_hat || !out) return IPTQ_ERR_NULL;
    if (n < 1) return IPTQ_ERR_SHAPE;
    if (mode != IPTQ_METRIC_LITERAL && mode != IPTQ_METRIC_PER_ELEMENT) return IPTQ_ERR_PARAM;
    if (!(op_count >= 0.0)) return IPTQ_ERR_PARAM;
    // sums in long double, element order: the inputs are at most a few 10^8 values of similar size
    long double signal = 0.0L, noise = 0.0L;
    for (int64_t i = 0; i < n; ++i) {
        const long double e = (long double)x[i] - (long double)x_hat[i];
        signal += (long double)x[i] * (long double)x[i];
        noise += e * e;
    }
    // Eq. 18.  The equation prints a factor 20 on the power ratio; the worked example of the same
    // section (power 10^4 against error powers 100 and 60: 20 dB and 22.21 dB) is 10 log10 of it,
    // and the example is what this follows.
    double q_db;
    if (noise == 0.0L) q_db = INFINITY;
    else if (signal == 0.0L) q_db = -INFINITY;
    else q_db = 10.0 * log10((double)(signal / noise));
    double p = (double)noise;                          // Eq. 19: || X - X^ ||_2^2
    double c = op_count;                               // Eq. 20
    if (mode == IPTQ_METRIC_PER_ELEMENT) { p /= (double)n; c /= (double)n; }
    const double nq = softplus(q_db), np = softplus(p), nc = softplus(c);
    const double inv_nq = isinf(nq) ? 0.0 : (nq == 0.0 ? INFINITY : 1.0 / nq);
    out->q_db = q_db; out->p = p; out->c = c;
    out->n_q = nq; out->n_p = np; out->n_c = nc;
    out->score = 3.0 / (inv_nq + np + nc);             // Eq. 16 for one layer
    return IPTQ_OK;
}

extern "C" int iptq_unified_select(const iptq_metric_t *candidates, int32_t n_candidates, int32_t *best)
{
    if (!candidates || !best) return IPTQ_ERR_NULL;
    if (n_candidates < 1) return IPTQ_ERR_SHAPE;
    int32_t b = 0;
    for (int32_t i = 1; i < n_candidates; ++i)
        if (candidates[i].score > candidates[b].score) b = i;
    *best = b;
    return IPTQ_OK;
}
