/*
 * TEST INFRASTRUCTURE - CPU oracle of the integer-only non-linear layers of IPTQ-ViT
 * (arXiv 2511.15369): dyadic requantization, the bit-shifting Softmax with the two
 * fractional-part approximations (Section 4.4, Eq. 6-15) and the polynomial GELU
 * (Section 4.3, Eq. 2, 3, 5).  Plain, scalar, single-threaded C with 64-bit
 * intermediates: one loop per step, in the paper's order, no blocking or fusion.
 *
 * Only the tests, the smoke check and the benchmark's cpu_baseline leg may use this
 * file.  It shares no code, header, table or helper with the HIP library and never
 * calls it; the HIP library never calls this.
 *
 * Conventions (the paper is silent on most of them; each is a declared reading):
 *   x >> k on a negative integer is the floor of x / 2^k (arithmetic shift);
 *   rshr_round(v, s) = floor((v + 2^(s-1)) / 2^s) for s >= 1 and v for s == 0
 *     (round to nearest, ties toward +infinity);
 *   the value INT32_MIN in a score row is "minus infinity": it never wins the row
 *     maximum, is never added to, and its exponential is 0; an entry INT32_MIN of an
 *     additive table (relative-position bias, shifted-window mask) makes the position
 *     minus infinity whatever the score is (any other entry is added with saturation);
 *   a row whose entries are all minus infinity yields the requantized value of 0.
 *
 * Parity pins: tests/test_oracle_*.py (closed forms, exact rational brackets,
 * shift / permutation invariance, float erf-GELU within the paper's error bound,
 * hand-worked rows under tests/golden/).  The defaults of the guard bits N, of M,
 * of the normalisation shift k and the mask semantics are not fixed by the paper:
 * parity unpinned for those choices (they are call parameters, not kernel code).
 */
#include <stdint.h>
#include <stdlib.h>

#define ORC_OK 0
#define ORC_ERR_ARG (-1)
#define ORC_ERR_NOMEM (-2)

typedef struct {
    int32_t m;    /* multiplier, |m| < 2^15 */
    int32_t s;    /* right shift, 0..62 */
    int32_t zp;   /* zero-point added after the shift */
    int32_t qmin; /* clip bounds of the target integer type */
    int32_t qmax;
} orc_dyadic;

typedef struct {
    int32_t variant;  /* 0: 1 + x/2 fractional part (Eq. 10); 1: 1 + (0.1011)b x (Eq. 13-14);
                         2: second-degree term of the Taylor series of Eq. 11 added to variant 1 */
    int32_t i0;       /* floor(1 / S_delta) (Eq. 14) */
    int32_t n_shift;  /* guard bits N: exponentials carry the scale S_delta / 2^N */
    int32_t m_bits;   /* M of Eq. 15 */
    int32_t out_bits; /* b of Eq. 15: probabilities on the scale 2^-(b-1) */
    int32_t pre_m;    /* optional requantization of the scores before the row max */
    int32_t pre_s;
    orc_dyadic post;  /* requantization of the b-bit probability */
    int32_t out_is_signed; /* 0: uint8 output, 1: int8 output */
} orc_softmax_params;

typedef struct {
    int32_t variant;   /* 0: degree 2 (Eq. 2 form); 1: degree 4 (Eq. 3) */
    int32_t q_b;       /* floor(b / S_e) < 0, S_e = S_in / sqrt 2 */
    int64_t q_c;       /* floor(1 / (a S_e^p)) < 0: the integer image of the constant 1 */
    int32_t k;         /* normalisation shift applied to 1 + L */
    int32_t zp_in;     /* zero-point of the input activation */
    int32_t max_abs_q; /* the centred input is clamped to [-max_abs_q, max_abs_q] */
    int32_t pre_m;     /* int32 entry only: requantization of the accumulator */
    int32_t pre_s;
    orc_dyadic post;   /* requantization of x * (1 + L) to the int8 output */
} orc_gelu_params;

/* ------------------------------------------------------------------ integer helpers */

static int64_t floor_div(int64_t a, int64_t b) /* b > 0 */
{
    int64_t q = a / b;
    if (a % b != 0 && a < 0) q -= 1;
    return q;
}

/* floor(v / 2^s): what ">>" means for two's-complement integers of either sign */
static int64_t shr_floor(int64_t v, int s)
{
    return floor_div(v, (int64_t)1 << s);
}

static int64_t rshr_round(int64_t v, int s)
{
    if (s == 0) return v;
    return shr_floor(v + ((int64_t)1 << (s - 1)), s);
}

static int64_t clamp64(int64_t v, int64_t lo, int64_t hi)
{
    if (v < lo) return lo;
    if (v > hi) return hi;
    return v;
}

static int64_t sat_i32(int64_t v)
{
    return clamp64(v, INT32_MIN, INT32_MAX);
}

/* y = clamp(rshr_round(x * m, s) + zp, qmin, qmax): multiply-then-shift requantization */
static int64_t requant1(int64_t x, const orc_dyadic *d)
{
    int64_t y = rshr_round(x * (int64_t)d->m, d->s) + (int64_t)d->zp;
    return clamp64(y, d->qmin, d->qmax);
}

static int dyadic_ok(const orc_dyadic *d, int out_is_signed)
{
    int64_t lo = out_is_signed ? -128 : 0, hi = out_is_signed ? 127 : 255;
    if (d->m <= -32768 || d->m >= 32768) return 0;
    if (d->s < 0 || d->s > 62) return 0;
    if (d->qmin > d->qmax || d->qmin < lo || d->qmax > hi) return 0;
    return 1;
}

static void store_out(void *out, int64_t idx, int64_t v, int out_is_signed)
{
    if (out_is_signed) ((int8_t *)out)[idx] = (int8_t)v;
    else ((uint8_t *)out)[idx] = (uint8_t)v;
}

/* ------------------------------------------------------------------ requantization */

int iptq_ref_requant(const int32_t *in, void *out, int64_t n, int32_t out_is_signed,
                     const orc_dyadic *d)
{
    if (n < 0 || !d || (n > 0 && (!in || !out))) return ORC_ERR_ARG;
    if (!dyadic_ok(d, out_is_signed)) return ORC_ERR_ARG;
    for (int64_t i = 0; i < n; ++i) store_out(out, i, requant1(in[i], d), out_is_signed);
    return ORC_OK;
}

/* ------------------------------------------------------------------ softmax */

/*
 * The integer exponential of one stabilised score delta <= 0 (Eq. 7-10, 13-14).
 * Returns Q_exp on the scale S_delta / 2^N.
 */
static int64_t bit_exp(int64_t delta, const orc_softmax_params *p)
{
    const int64_t i0 = p->i0;
    /* Eq. 7: multiply by log2(e) ~ (1.0111)b with shifts */
    int64_t qp = delta + shr_floor(delta, 1) - shr_floor(delta, 4);
    /* Eq. 8: S qp = -q + S (-r), 0 <= r < i0 */
    int64_t n = -qp;
    int64_t q = n / i0;
    int64_t r = n - q * i0;
    /* fractional part 2^(S (-r)) on the integer scale 1/S ~ i0 */
    int64_t frac;
    if (p->variant == 0)
        frac = shr_floor(-r, 1); /* Eq. 10: x / 2 */
    else
        frac = shr_floor(-r, 1) + shr_floor(-r, 3) + shr_floor(-r, 4); /* Eq. 13: Phi(x) */
    /* Eq. 11 with D = 2 (the "D2" form of the degree ablation; its integer form is not printed:
       declared reading): y = Phi(-r) is ln2 X on the scale 1/S ~ i0, so (ln2 X)^2 / 2 on that
       scale is y^2 / (2 i0), floored */
    if (p->variant == 2) frac += floor_div(frac * frac, 2 * i0);
    int64_t base = frac + i0; /* Eq. 14: Phi(-r) + floor(1 / S) */
    /* Eq. 9: the integer part is a right shift; a shift of 32 or more leaves nothing */
    if (q >= 32) return 0;
    return shr_floor(base * ((int64_t)1 << p->n_shift), (int)q);
}

static int softmax_params_ok(const orc_softmax_params *p, int32_t cols)
{
    if (p->variant != 0 && p->variant != 1 && p->variant != 2) return 0;
    if (p->i0 < 16 || p->i0 >= (1 << 24)) return 0;
    if (p->variant == 2 && p->i0 >= (1 << 16)) return 0; /* y^2 stays below 2^31 */
    if (p->n_shift < 0 || p->n_shift > 20) return 0;
    if (((int64_t)p->i0 << p->n_shift) >= (1 << 24)) return 0;
    if (p->out_bits < 2 || p->out_bits > 8) return 0;
    if (p->m_bits < p->out_bits - 1 || p->m_bits > 31) return 0;
    if ((int64_t)cols * ((int64_t)p->i0 << p->n_shift) > ((int64_t)1 << p->m_bits)) return 0;
    if (p->pre_m < 1 || p->pre_m >= 32768 || p->pre_s < 0 || p->pre_s > 62) return 0;
    if (p->out_is_signed != 0 && p->out_is_signed != 1) return 0;
    return dyadic_ok(&p->post, p->out_is_signed);
}

/* x + t for one entry t of an additive table: minus infinity if either is */
static int64_t add_table_entry(int64_t x, int64_t t)
{
    if (x == INT32_MIN || t == INT32_MIN) return INT32_MIN;
    return sat_i32(x + t);
}

/*
 * Rows are ordered [image, window, head, query].  bias: [bias_period_rows, cols], row r takes
 * table row r mod bias_period_rows (the relative-position bias, period heads * cols).
 * mask: [n_windows, cols, cols], the shifted-window mask: row r lies in window
 * (r div (heads * cols)) mod n_windows and is query r mod cols of it.  Either may be NULL.
 */
int iptq_ref_softmax_i32_windowed(const int32_t *scores, const int32_t *bias,
                                  int64_t bias_period_rows, const int32_t *mask,
                                  int64_t n_windows, int64_t heads, void *out, int64_t rows,
                                  int32_t cols, const orc_softmax_params *p)
{
    if (rows < 0 || cols < 1 || !p) return ORC_ERR_ARG;
    if (rows > 0 && (!scores || !out)) return ORC_ERR_ARG;
    if (bias && bias_period_rows < 1) return ORC_ERR_ARG;
    if (mask && (n_windows < 1 || heads < 1)) return ORC_ERR_ARG;
    if (!softmax_params_ok(p, cols)) return ORC_ERR_ARG;

    int64_t *x = (int64_t *)malloc(sizeof(int64_t) * (size_t)cols);
    int64_t *qexp = (int64_t *)malloc(sizeof(int64_t) * (size_t)cols);
    if (!x || !qexp) { free(x); free(qexp); return ORC_ERR_NOMEM; }

    const int has_pre = !(p->pre_m == 1 && p->pre_s == 0);
    for (int64_t row = 0; row < rows; ++row) {
        const int32_t *srow = scores + row * cols;
        const int32_t *brow = bias ? bias + (row % bias_period_rows) * cols : 0;
        const int32_t *mrow = 0;
        if (mask) {
            const int64_t window = (row / (heads * cols)) % n_windows;
            const int64_t query = row % cols;
            mrow = mask + (window * cols + query) * cols;
        }

        /* additive bias, additive mask and optional requantization; minus infinity stays as it is */
        for (int32_t j = 0; j < cols; ++j) {
            int64_t v = srow[j];
            if (brow) v = add_table_entry(v, brow[j]);
            if (mrow) v = add_table_entry(v, mrow[j]);
            if (v != INT32_MIN && has_pre) v = sat_i32(rshr_round(v * (int64_t)p->pre_m, p->pre_s));
            x[j] = v;
        }

        /* Eq. 6: row maximum */
        int64_t mx = INT32_MIN;
        for (int32_t j = 0; j < cols; ++j)
            if (x[j] > mx) mx = x[j];

        /* exponentials and their sum (denominator of Eq. 15) */
        int64_t sum = 0;
        for (int32_t j = 0; j < cols; ++j) {
            if (x[j] == INT32_MIN) { qexp[j] = 0; continue; }
            int64_t delta = x[j] - mx;                      /* Eq. 6 */
            if (delta < -((int64_t)1 << 30)) delta = -((int64_t)1 << 30);
            qexp[j] = bit_exp(delta, p);
            sum += qexp[j];
        }

        /* Eq. 15: IntDiv */
        int64_t f = sum > 0 ? (((int64_t)1 << p->m_bits) / sum) : 0;
        for (int32_t j = 0; j < cols; ++j) {
            int64_t prob = shr_floor(f * qexp[j], p->m_bits - (p->out_bits - 1));
            store_out(out, row * cols + j, requant1(prob, &p->post), p->out_is_signed);
        }
    }
    free(x);
    free(qexp);
    return ORC_OK;
}

int iptq_ref_softmax_i32(const int32_t *scores, const int32_t *bias, int64_t bias_period_rows,
                         void *out, int64_t rows, int32_t cols, const orc_softmax_params *p)
{
    return iptq_ref_softmax_i32_windowed(scores, bias, bias_period_rows, 0, 0, 0, out, rows, cols, p);
}

/* ------------------------------------------------------------------ GELU */

static int gelu_params_ok(const orc_gelu_params *p)
{
    if (p->variant != 0 && p->variant != 1) return 0;
    if (p->q_b >= 0 || p->q_c >= 0) return 0;
    if (p->k < 0 || p->k > 62) return 0;
    if (p->max_abs_q < 1) return 0;
    if (p->pre_m < 1 || p->pre_m >= 32768 || p->pre_s < 0 || p->pre_s > 62) return 0;
    /* |q_b|^p + 2|q_c| must stay inside int64 and q * v inside int32: |v| is at most that sum
       divided by 2^k and rounded UP (a negative numerator is floored away from zero) */
    const int64_t lim = (int64_t)1 << 62;
    int64_t t = -(int64_t)p->q_b;
    if (t > ((int64_t)1 << 30)) return 0;
    int64_t tp = t * t;
    if (p->variant == 1) {
        if (t >= ((int64_t)1 << 15)) return 0;
        tp = tp * tp;
    }
    if (-p->q_c >= lim / 4 || tp >= lim / 2) return 0;
    int64_t vmax = (tp + 2 * (-p->q_c) + (((int64_t)1 << p->k) - 1)) >> p->k;
    if (vmax >= ((int64_t)1 << 31)) return 0;
    if (vmax * (int64_t)p->max_abs_q >= ((int64_t)1 << 31)) return 0;
    return dyadic_ok(&p->post, 1);
}

/* one centred, already requantized input value -> int8 code */
static int64_t gelu_elem(int64_t in, const orc_gelu_params *p)
{
    int64_t q = clamp64(in - (int64_t)p->zp_in, -(int64_t)p->max_abs_q, (int64_t)p->max_abs_q);
    int64_t sgn = (q > 0) - (q < 0);
    int64_t aq = q < 0 ? -q : q;
    /* Eq. 3: clip |x| at -b, then add b: t in [q_b, 0] */
    int64_t nb = -(int64_t)p->q_b;
    int64_t t = (aq < nb ? aq : nb) + (int64_t)p->q_b;
    /* t^p, reusing the square for the quartic */
    int64_t tp = t * t;
    if (p->variant == 1) tp = tp * tp;
    /* a (.)^p + 1 on the integer scale where 1 is q_c; times sign; plus the 1 of Eq. 5 */
    int64_t u = tp + p->q_c;
    int64_t v = shr_floor(sgn * u + p->q_c, p->k);
    /* Eq. 5: x * (1 + L); the factor 1/2 lives in the output scale */
    int64_t w = q * v;
    return requant1(w, &p->post);
}

int iptq_ref_gelu_i8(const int8_t *in, int8_t *out, int64_t n, const orc_gelu_params *p)
{
    if (n < 0 || !p || (n > 0 && (!in || !out))) return ORC_ERR_ARG;
    if (!gelu_params_ok(p)) return ORC_ERR_ARG;
    for (int64_t i = 0; i < n; ++i) out[i] = (int8_t)gelu_elem(in[i], p);
    return ORC_OK;
}

int iptq_ref_gelu_i32(const int32_t *in, int8_t *out, int64_t n, const orc_gelu_params *p)
{
    if (n < 0 || !p || (n > 0 && (!in || !out))) return ORC_ERR_ARG;
    if (!gelu_params_ok(p)) return ORC_ERR_ARG;
    const int has_pre = !(p->pre_m == 1 && p->pre_s == 0);
    for (int64_t i = 0; i < n; ++i) {
        int64_t v = in[i];
        if (has_pre) v = sat_i32(rshr_round(v * (int64_t)p->pre_m, p->pre_s));
        out[i] = (int8_t)gelu_elem(v, p);
    }
    return ORC_OK;
}

/* intermediate values of one softmax exponential, for tests that check each step */
int64_t iptq_ref_bit_exp(int64_t delta, const orc_softmax_params *p)
{
    return bit_exp(delta, p);
}

/* the same for an array of deltas */
int iptq_ref_bit_exp_array(const int64_t *delta, int64_t *out, int64_t n, const orc_softmax_params *p)
{
    if (n < 0 || !p || (n > 0 && (!delta || !out))) return ORC_ERR_ARG;
    if (!softmax_params_ok(p, 1)) return ORC_ERR_ARG;
    for (int64_t i = 0; i < n; ++i) out[i] = bit_exp(delta[i] < -((int64_t)1 << 30) ? -((int64_t)1 << 30) : delta[i], p);
    return ORC_OK;
}
