// Host-side validation and constant derivation.  No HIP calls here: every error other
// than IPTQ_ERR_HIP is decided in this file, before anything is enqueued.
#include "plan.h"

#include <math.h>
#include <string.h>

namespace iptq {

static int bitlen64(uint64_t v)
{
    int n = 0;
    while (v) { ++n; v >>= 1; }
    return n;
}

bool make_magic_u32(uint32_t d, int nbits, uint32_t *magic, int32_t *sh)
{
    if (d < 2 || nbits < 1 || nbits > 31) return false;
    if (bitlen64(d) > nbits) return false;
    int l = bitlen64((uint64_t)d - 1);  // ceil(log2 d)
    int extra = nbits + l - 32;
    if (extra < 0) extra = 0;
    const int w = 32 + extra;  // <= 63 + ... : nbits <= 31 and l <= 31 give w <= 62
    unsigned __int128 two_w = (unsigned __int128)1 << w;
    unsigned __int128 mg = two_w / d + 1;
    if (mg >> 32) return false;
    // error term e = mg * d - 2^w must satisfy 0 < e <= d, and 2^nbits * e <= 2^w
    unsigned __int128 e = mg * d - two_w;
    if (e == 0 || e > d) return false;
    if (((unsigned __int128)e << nbits) > two_w) return false;
    *magic = (uint32_t)mg;
    *sh = extra;
    return true;
}

int64_t neg_qp_of(int64_t d)
{
    // delta = -d:  -(delta + (delta >> 1) - (delta >> 4)) with floor shifts
    return d + ((d + 1) >> 1) - ((d + 15) >> 4);
}

int check_dyadic(const iptq_dyadic_t *p, int out_is_signed)
{
    if (!p) return IPTQ_ERR_NULL;
    if (out_is_signed != 0 && out_is_signed != 1) return IPTQ_ERR_PARAM;
    const int32_t lo = out_is_signed ? -128 : 0, hi = out_is_signed ? 127 : 255;
    if (p->m <= -32768 || p->m >= 32768) return IPTQ_ERR_PARAM;
    if (p->s < 0 || p->s > 62) return IPTQ_ERR_PARAM;
    if (p->zp < -(1 << 24) || p->zp > (1 << 24)) return IPTQ_ERR_PARAM;
    if (p->qmin > p->qmax || p->qmin < lo || p->qmax > hi) return IPTQ_ERR_PARAM;
    return IPTQ_OK;
}

int plan_requant(const iptq_dyadic_t *p, int out_is_signed, DyadicDev *out)
{
    int rc = check_dyadic(p, out_is_signed);
    if (rc != IPTQ_OK) return rc;
    out->m = p->m; out->s = p->s; out->zp = p->zp; out->qmin = p->qmin; out->qmax = p->qmax;
    return IPTQ_OK;
}

int plan_softmax(const iptq_softmax_params_t *p, int64_t rows, int32_t cols, int has_bias,
                 int64_t bias_period_rows, SoftmaxDev *out)
{
    if (!p) return IPTQ_ERR_NULL;
    if (rows < 0 || rows >= ((int64_t)1 << 31)) return IPTQ_ERR_SHAPE;
    if (cols < 1 || cols > IPTQ_COLS_MAX) return IPTQ_ERR_SHAPE;
    if (has_bias && (bias_period_rows < 1 || bias_period_rows >= ((int64_t)1 << 31)))
        return IPTQ_ERR_SHAPE;
    if (p->variant != IPTQ_SOFTMAX_SHIFT_LINEAR && p->variant != IPTQ_SOFTMAX_EFFICIENT_BITEXP &&
        p->variant != IPTQ_SOFTMAX_BITEXP_DEGREE2)
        return IPTQ_ERR_PARAM;
    if (p->algo != IPTQ_ALGO_AUTO && p->algo != IPTQ_ALGO_GENERIC &&
        p->algo != IPTQ_ALGO_DYNAMIC && p->algo != IPTQ_ALGO_WIDE && p->algo != IPTQ_ALGO_SLAB)
        return IPTQ_ERR_PARAM;
    if (p->i0 < 16 || p->i0 >= (1 << 24)) return IPTQ_ERR_PARAM;
    if (p->n_shift < 0 || p->n_shift > 20) return IPTQ_ERR_PARAM;
    if (((int64_t)p->i0 << p->n_shift) >= (1 << 24)) return IPTQ_ERR_PARAM;
    if (p->out_bits < 2 || p->out_bits > 8) return IPTQ_ERR_PARAM;
    if (p->m_bits < p->out_bits - 1 || p->m_bits > 31) return IPTQ_ERR_PARAM;
    if (p->pre_m < 1 || p->pre_m >= 32768 || p->pre_s < 0 || p->pre_s > 62) return IPTQ_ERR_PARAM;
    if (p->out_is_signed != 0 && p->out_is_signed != 1) return IPTQ_ERR_PARAM;
    int rc = check_dyadic(&p->post, p->out_is_signed);
    if (rc != IPTQ_OK) return rc;
    const int64_t i0n = (int64_t)p->i0 << p->n_shift;
    if ((int64_t)cols * i0n > ((int64_t)1 << p->m_bits)) return IPTQ_ERR_RANGE;
    // second-degree form: the square of Phi(-r) (|Phi| < 0.6875 i0) must stay below 2^31
    if (p->variant == IPTQ_SOFTMAX_BITEXP_DEGREE2 && p->i0 >= (1 << 16)) return IPTQ_ERR_RANGE;

    // Deltas at or below -D shift every bit of (base << N) out: q >= bitlen(i0 << N).
    // n(d) grows by 1 or 2 per step of d (< i0), so the first such d has q == L exactly.
    const int L = bitlen64((uint64_t)i0n);
    int64_t lo = 0, hi = (int64_t)1 << 30;
    const int64_t want = (int64_t)L * p->i0;
    while (lo < hi) {
        int64_t mid = lo + (hi - lo) / 2;
        if (neg_qp_of(mid) >= want) hi = mid; else lo = mid + 1;
    }
    const int64_t D = lo;
    const int64_t n_max = neg_qp_of(D);
    const int64_t q_at_d = n_max / p->i0;
    if (q_at_d < L || q_at_d > 31 || D >= ((int64_t)1 << 30)) return IPTQ_ERR_RANGE;
    uint32_t magic; int32_t sh;
    if (!make_magic_u32((uint32_t)p->i0, bitlen64((uint64_t)n_max), &magic, &sh))
        return IPTQ_ERR_RANGE;
    // spot check of the divider at every multiple of i0 in range and its neighbours
    for (int64_t kq = 0; kq <= q_at_d + 1; ++kq) {
        for (int64_t dn = -1; dn <= 1; ++dn) {
            int64_t n = kq * p->i0 + dn;
            if (n < 0 || n > n_max) continue;
            uint64_t got = (((uint64_t)n * magic) >> 32) >> sh;
            if ((int64_t)got != n / p->i0) return IPTQ_ERR_RANGE;
        }
    }

    memset(out, 0, sizeof(*out));
    out->i0 = p->i0;
    out->i0n = (int32_t)i0n;
    out->n_shift = p->n_shift;
    out->magic = magic;
    out->magic_sh = sh;
    out->d_clamp = (int32_t)D;
    out->m_bits = p->m_bits;
    out->p_shift = p->m_bits - (p->out_bits - 1);
    out->pre_m = p->pre_m; out->pre_s = p->pre_s;
    if (p->pre_m == 1 && p->pre_s == 0) {
        out->pre_mode = 0;
    } else if (p->pre_s >= 16) {
        // (x m + 2^(s-1)) >> s == (x m 2^(32-s) + 2^31) >> 32 for s <= 32, and
        // ((x m + 2^(s-1)) >> 32) >> (s - 32) beyond; |x m| < 2^46, so the result fits 32 bits
        out->pre_mode = 1;
        out->pre_mul = p->pre_s <= 32 ? p->pre_m << (32 - p->pre_s) : p->pre_m;
        out->pre_rnd = p->pre_s <= 32 ? ((int64_t)1 << 31) : ((int64_t)1 << (p->pre_s - 1));
        out->pre_sh2 = p->pre_s <= 32 ? 0 : p->pre_s - 32;
    } else {
        out->pre_mode = 2;
    }
    out->post_m = p->post.m; out->post_s = p->post.s; out->post_zp = p->post.zp;
    out->qmin = p->post.qmin; out->qmax = p->post.qmax;
    out->post_xor = (p->out_is_signed == 1 && p->post.m == 1 && p->post.s == 0 && p->post.zp == -128 &&
                     p->post.qmin == -128 && p->post.qmax >= 0) ? 0x80808080u : 0u;
    out->variant = p->variant;
    out->d2_magic = 0;
    out->d2_sh = 0;
    if (p->variant == IPTQ_SOFTMAX_BITEXP_DEGREE2 &&
        !make_magic_u32((uint32_t)(2 * p->i0), 31, &out->d2_magic, &out->d2_sh))
        return IPTQ_ERR_RANGE;
    // Packed 16-bit path: clamped delta, n and (i0 << N) must fit 16 bits, the per-row factor
    // shifted to the top byte must fit 24 bits, and a 24-bit divider multiplier must be exact.
    out->mode16 = 0;
    out->mg24 = 0;
    out->t16 = 0;
    if (D <= 32767 && i0n < (1 << 15) && out->p_shift <= 24 && i0n >= ((int64_t)1 << p->out_bits)) {
        for (int t = 0; t <= 12; ++t) {
            const uint64_t two = (uint64_t)1 << (32 - t);
            const uint64_t mg = two / (uint64_t)p->i0 + 1;
            if (mg >= ((uint64_t)1 << 24)) continue;
            const uint64_t e = mg * (uint64_t)p->i0 - two;      // 0 < e <= i0
            const bool fits = ((uint64_t)n_max << t) <= 65535;
            const bool exact = e > 0 && e <= (uint64_t)p->i0 && (uint64_t)n_max * e < two;
            if (fits && exact) {
                out->mode16 = t == 0 ? 1 : 2;
                out->mg24 = (uint32_t)mg;
                out->t16 = t;
            }
            break;
        }
    }
    out->pre_rowconst = 0;
    out->pre_dmax = 0;
    // (the folded requantization is instantiated for the first-degree exponentials only)
    if (out->pre_mode == 1 && out->mode16 != 0 && p->pre_s <= 31 && p->variant != IPTQ_SOFTMAX_BITEXP_DEGREE2) {
        const int64_t two_s = (int64_t)1 << p->pre_s;
        const int64_t dmax = (D * two_s + p->pre_m - 1) / p->pre_m;
        if (dmax < ((int64_t)1 << 24) && dmax * p->pre_m + two_s <= ((int64_t)1 << 32)) {
            out->pre_rowconst = 1;
            out->pre_dmax = (uint32_t)dmax;
        }
    }
    out->bias_period_rows = has_bias ? (int32_t)bias_period_rows : 1;
    out->period_magic = 0;
    out->period_sh = 0;
    if (has_bias && bias_period_rows >= 2) {
        if (!make_magic_u32((uint32_t)bias_period_rows, 31, &out->period_magic, &out->period_sh))
            return IPTQ_ERR_RANGE;
    }
    return IPTQ_OK;
}

int plan_softmax_mask(int64_t n_windows, int64_t heads, int32_t cols, SoftmaxDev *out)
{
    if (n_windows < 1 || heads < 1) return IPTQ_ERR_SHAPE;
    const int64_t group = heads * (int64_t)cols;
    if (heads >= ((int64_t)1 << 31) || n_windows >= ((int64_t)1 << 31) ||
        group >= ((int64_t)1 << 31) || group * n_windows >= ((int64_t)1 << 31) ||
        n_windows * (int64_t)cols * cols >= ((int64_t)1 << 31))
        return IPTQ_ERR_SHAPE;
    out->n_windows = (int32_t)n_windows;
    out->group_rows = (int32_t)group;
    out->mask_period_rows = (int32_t)(group * n_windows);
    out->mperiod_magic = out->group_magic = 0;
    out->mperiod_sh = out->group_sh = 0;
    if (out->mask_period_rows >= 2 &&
        !make_magic_u32((uint32_t)out->mask_period_rows, 31, &out->mperiod_magic, &out->mperiod_sh))
        return IPTQ_ERR_RANGE;
    if (group >= 2 && !make_magic_u32((uint32_t)group, 31, &out->group_magic, &out->group_sh))
        return IPTQ_ERR_RANGE;
    return IPTQ_OK;
}

int plan_gelu(const iptq_gelu_params_t *p, int is_i8_entry, GeluDev *out)
{
    if (!p) return IPTQ_ERR_NULL;
    if (p->variant != IPTQ_GELU_POLY2 && p->variant != IPTQ_GELU_POLY4_DATA_AWARE)
        return IPTQ_ERR_PARAM;
    if (p->algo != IPTQ_ALGO_AUTO && p->algo != IPTQ_ALGO_GENERIC) return IPTQ_ERR_PARAM;
    if (p->q_b >= 0 || p->q_c >= 0) return IPTQ_ERR_PARAM;
    if (p->k < 0 || p->k > 62) return IPTQ_ERR_PARAM;
    if (p->max_abs_q < 1) return IPTQ_ERR_PARAM;
    if (p->pre_m < 1 || p->pre_m >= 32768 || p->pre_s < 0 || p->pre_s > 62) return IPTQ_ERR_PARAM;
    if (is_i8_entry && (p->zp_in < -128 || p->zp_in > 128)) return IPTQ_ERR_PARAM;
    int rc = check_dyadic(&p->post, 1);
    if (rc != IPTQ_OK) return rc;
    const int quartic = p->variant == IPTQ_GELU_POLY4_DATA_AWARE;
    const int64_t t = -(int64_t)p->q_b;
    if (t > ((int64_t)1 << 30)) return IPTQ_ERR_RANGE;
    if (quartic && t >= (1 << 15)) return IPTQ_ERR_RANGE;
    int64_t tp = t * t;
    if (quartic) tp *= tp;
    if (tp >= ((int64_t)1 << 61) || -p->q_c >= ((int64_t)1 << 60)) return IPTQ_ERR_RANGE;
    // |v| <= ceil((|q_b|^p + 2|q_c|) / 2^k): a negative numerator is floored away from zero
    const int64_t vmax = (tp + 2 * (-p->q_c) + (((int64_t)1 << p->k) - 1)) >> p->k;
    if (vmax >= ((int64_t)1 << 31)) return IPTQ_ERR_RANGE;
    if (vmax * (int64_t)p->max_abs_q >= ((int64_t)1 << 31)) return IPTQ_ERR_RANGE;
    out->quartic = quartic;
    out->q_b = p->q_b; out->q_c = p->q_c; out->k = p->k; out->zp_in = p->zp_in;
    out->max_abs_q = p->max_abs_q;
    out->pre_m = p->pre_m; out->pre_s = p->pre_s;
    out->post_m = p->post.m; out->post_s = p->post.s; out->post_zp = p->post.zp;
    out->qmin = p->post.qmin; out->qmax = p->post.qmax;
    out->fast = (p->post.s >= 16 && t <= 46340) ? 1 : 0;
    out->pre_mode = (p->pre_m == 1 && p->pre_s == 0) ? 0 : (p->pre_s >= 15 ? 1 : 2);
    return IPTQ_OK;
}

}  // namespace iptq

// ------------------------------------------------------------------ C ABI: host helpers

extern "C" int iptq_version(void) { return 200; }   // 0.2.0: window masks, second-degree exponential, Unified Metric

extern "C" const char *iptq_strerror(int code)
{
    switch (code) {
    case IPTQ_OK: return "ok";
    case IPTQ_ERR_NULL: return "a required pointer is NULL";
    case IPTQ_ERR_SHAPE: return "invalid shape (negative count, cols out of range, or rows >= 2^31)";
    case IPTQ_ERR_PARAM: return "a parameter is outside its documented domain";
    case IPTQ_ERR_RANGE: return "parameters could overflow the fixed-width integer path";
    case IPTQ_ERR_HIP: return "the HIP runtime refused the launch";
    case IPTQ_ERR_ALIGN: return "a pointer is not aligned to its element type";
    default: return "unknown iptq error code";
    }
}

extern "C" int iptq_make_dyadic(double ratio, int32_t *m, int32_t *s)
{
    if (!m || !s) return IPTQ_ERR_NULL;
    const double a = fabs(ratio);
    if (!(a > 0.0) || isinf(a)) return IPTQ_ERR_PARAM;
    int e = 0;
    const double f = frexp(a, &e);                 // a = f * 2^e, f in [0.5, 1)
    int64_t mm = (int64_t)floor(f * 32768.0 + 0.5);
    int64_t ss = 15 - (int64_t)e;
    if (mm == 32768) { mm = 16384; ss -= 1; }
    if (ss > 62) { mm = (int64_t)floor(ldexp(a, 62) + 0.5); ss = 62; }
    if (ss < 0) return IPTQ_ERR_RANGE;
    *m = (int32_t)(ratio < 0 ? -mm : mm);
    *s = (int32_t)ss;
    return IPTQ_OK;
}

extern "C" int iptq_softmax_prepare(double s_delta, int32_t cols, int32_t variant,
                                    int32_t out_is_signed, iptq_softmax_params_t *out)
{
    if (!out) return IPTQ_ERR_NULL;
    if (!(s_delta > 0.0) || isinf(s_delta)) return IPTQ_ERR_PARAM;
    if (cols < 1 || cols > IPTQ_COLS_MAX) return IPTQ_ERR_SHAPE;
    if (variant != 0 && variant != 1 && variant != 2) return IPTQ_ERR_PARAM;
    const double inv = floor(1.0 / s_delta);
    if (inv < 16.0 || inv >= 16777216.0) return IPTQ_ERR_RANGE;
    if (variant == 2 && inv >= 65536.0) return IPTQ_ERR_RANGE;
    const int32_t i0 = (int32_t)inv;
    int n = 15 - iptq::bitlen64((uint64_t)i0);
    if (n < 0) n = 0;
    const int m_bits = 30;
    while (n > 0 && (int64_t)cols * ((int64_t)i0 << n) > ((int64_t)1 << m_bits)) --n;
    memset(out, 0, sizeof(*out));
    out->variant = variant;
    out->i0 = i0;
    out->n_shift = n;
    out->m_bits = m_bits;
    out->out_bits = 8;
    out->pre_m = 1; out->pre_s = 0;
    out->post.m = 1; out->post.s = 0; out->post.zp = 0; out->post.qmin = 0;
    out->post.qmax = out_is_signed ? 127 : 255;
    out->out_is_signed = out_is_signed ? 1 : 0;
    out->algo = IPTQ_ALGO_AUTO;
    return IPTQ_OK;
}

extern "C" int iptq_gelu_prepare(double s_in, double s_out, int32_t zp_in, int32_t zp_out,
                                 int32_t variant, int32_t max_abs_q, iptq_gelu_params_t *out)
{
    if (!out) return IPTQ_ERR_NULL;
    if (!(s_in > 0.0) || !(s_out > 0.0) || isinf(s_in) || isinf(s_out)) return IPTQ_ERR_PARAM;
    if (variant != 0 && variant != 1) return IPTQ_ERR_PARAM;
    if (max_abs_q < 1) return IPTQ_ERR_PARAM;
    // erf polynomial a (x + b)^p + 1: quartic coefficients from Section 4.3; the second-order
    // ones are the I-BERT fit that Eq. 2 refers to
    const int p = variant == 1 ? 4 : 2;
    const double a = variant == 1 ? -0.019913 : -0.2888;
    const double b = variant == 1 ? -2.698088 : -1.769;
    const double s_e = s_in / sqrt(2.0);
    const double qb = floor(b / s_e);
    const double sq = s_e * s_e;
    const double s_l = a * (p == 2 ? sq : sq * sq);
    const double qc = floor(1.0 / s_l);
    if (qb <= -1073741824.0 || (p == 4 && qb <= -32768.0)) return IPTQ_ERR_RANGE;
    if (qc <= -1152921504606846976.0) return IPTQ_ERR_RANGE;
    const int64_t q_b = (int64_t)qb, q_c = (int64_t)qc;
    int64_t tp = q_b * q_b;
    if (p == 4) tp *= tp;
    const int64_t vmax = tp + 2 * (-q_c);
    int k = 0;
    // smallest k with ceil(vmax / 2^k) * max_abs_q < 2^31 (|v| can reach the ceiling)
    auto v_bound = [&](int kk) { return (unsigned __int128)((vmax + (((int64_t)1 << kk) - 1)) >> kk); };
    while (k < 62 && v_bound(k) * (unsigned __int128)max_abs_q >= ((unsigned __int128)1 << 31)) ++k;
    const double ratio = ((s_in * s_l) * ldexp(1.0, k) / 2.0) / s_out;
    int32_t m = 0, s = 0;
    int rc = iptq_make_dyadic(ratio, &m, &s);
    if (rc != IPTQ_OK) return rc;
    memset(out, 0, sizeof(*out));
    out->variant = variant;
    out->q_b = (int32_t)q_b;
    out->q_c = q_c;
    out->k = k;
    out->zp_in = zp_in;
    out->max_abs_q = max_abs_q;
    out->pre_m = 1; out->pre_s = 0;
    out->post.m = m; out->post.s = s; out->post.zp = zp_out; out->post.qmin = -128;
    out->post.qmax = 127;
    out->algo = IPTQ_ALGO_AUTO;
    return IPTQ_OK;
}
