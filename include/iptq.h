/*
 * iptq.h - C ABI of the MI355X (gfx950) integer-only non-linear layers of IPTQ-ViT
 * (arXiv 2511.15369): bit-shifting Softmax (Section 4.4), polynomial GELU (Section 4.3)
 * and the dyadic multiply-then-shift requantization around both.
 *
 * General rules of every entry point
 *   - Pointers named d_* are DEVICE pointers owned by the caller; the library never
 *     allocates, frees or retains them.  Parameter structs are HOST pointers and are
 *     copied before the call returns.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue work: they return before the kernels finish and never synchronise.
 *   - Return value: IPTQ_OK (0) or a negative IPTQ_ERR_* code.  All argument checks run
 *     on the host before anything is enqueued: on an error other than IPTQ_ERR_HIP no
 *     kernel was launched and the outputs are untouched.
 *   - The library keeps no state; calls on different streams may overlap freely as long
 *     as their output buffers do not.
 *   - Arithmetic conventions: x >> k on a negative integer is floor(x / 2^k);
 *     rshr_round(v, s) = (v + 2^(s-1)) >> s for s >= 1 and v for s == 0 (ties go up).
 *   - The kernels contain integer instructions only (no floating point, no matrix cores).
 */
#ifndef IPTQ_H
#define IPTQ_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define IPTQ_OK 0
#define IPTQ_ERR_NULL (-1)  /* a required pointer is NULL */
#define IPTQ_ERR_SHAPE (-2) /* negative count, cols outside [1, IPTQ_COLS_MAX], rows >= 2^31 */
#define IPTQ_ERR_PARAM (-3) /* a parameter is outside its documented domain */
#define IPTQ_ERR_RANGE (-4) /* parameters are valid one by one but could overflow the fixed-width path */
#define IPTQ_ERR_HIP (-5)   /* the HIP runtime refused the launch */
#define IPTQ_ERR_ALIGN (-6) /* a pointer is not aligned to its element type */

#define IPTQ_COLS_MAX 65536

/* Softmax fractional-part approximation of 2^(S(-r)) (the per-layer choice of Section 4.2) */
#define IPTQ_SOFTMAX_SHIFT_LINEAR 0     /* 1 + x/2            (Eq. 10) */
#define IPTQ_SOFTMAX_EFFICIENT_BITEXP 1 /* 1 + (0.1011)b x    (Eq. 12-14) */
#define IPTQ_SOFTMAX_BITEXP_DEGREE2 2   /* 1 + y + y^2/2, y = (0.1011)b x: Eq. 11 with D = 2, the
                                           second-degree form of the degree ablation (Section 4.4) */
/* GELU erf polynomial */
#define IPTQ_GELU_POLY2 0            /* second order a(x+b)^2 + c form (Eq. 2) */
#define IPTQ_GELU_POLY4_DATA_AWARE 1 /* quartic, a = -0.019913, b = -2.698088 (Eq. 3) */

/* algo field: which kernel family serves the call (results are identical) */
#define IPTQ_ALGO_AUTO 0
#define IPTQ_ALGO_GENERIC 1 /* softmax: one wavefront per row, any cols; GELU: polynomial per element */
#define IPTQ_ALGO_DYNAMIC 2 /* softmax only: the register-resident kernel with run-time row length
                               (rows up to about 635 scores), also where a compiled row length
                               would serve */
#define IPTQ_ALGO_WIDE 3    /* softmax only: one wavefront (rows up to 4096 scores) or one workgroup
                               (up to 40957) per row, row in registers, no LDS staging, also where
                               another kernel would serve */
#define IPTQ_ALGO_SLAB 4    /* softmax only: the slab kernels (compiled row length if there is one,
                               else run-time row length) also for a call of few rows, which
                               IPTQ_ALGO_AUTO gives to one wavefront per row */

/*
 * y = clamp(rshr_round(x * m, s) + zp, qmin, qmax)
 * |m| < 2^15, 0 <= s <= 62, qmin <= qmax inside the output type ([0,255] or [-128,127]).
 */
typedef struct {
    int32_t m;
    int32_t s;
    int32_t zp;
    int32_t qmin;
    int32_t qmax;
} iptq_dyadic_t;

/*
 * Integer softmax of one row x[0..cols) of int32 scores (Section 4.4):
 *   0. x_j == INT32_MIN means "minus infinity" (masked) at every stage below; an entry
 *      INT32_MIN of an additive table (bias, window mask) makes x_j minus infinity whatever
 *      the score; otherwise x_j = sat32(x_j + entry) for each table given, then
 *      x_j = sat32(rshr_round(x_j * pre_m, pre_s)) unless (pre_m, pre_s) == (1, 0)
 *   1. d_j = max(x_j - max_j x_j, -2^30)                                  (Eq. 6)
 *   2. Qp = d + (d >> 1) - (d >> 4)                                       (Eq. 7)
 *   3. n = -Qp, q = n div i0, r = n mod i0                                (Eq. 8)
 *   4. base = i0 + ((-r) >> 1)                       variant 0            (Eq. 10)
 *      base = i0 + ((-r) >> 1) + ((-r) >> 3) + ((-r) >> 4)  variant 1     (Eq. 13-14)
 *      base = i0 + y + floor(y^2 / (2 i0)), y the variant-1 sum   variant 2 (Eq. 11, D = 2; the
 *      paper prints no integer form of it: this one is the library's reading; i0 < 2^16)
 *   5. Qexp_j = 0 if masked or q >= 32, else (base << n_shift) >> q       (Eq. 9)
 *   6. f = floor(2^m_bits / sum_j Qexp_j)  (0 for an all-masked row)
 *      p_j = (f * Qexp_j) >> (m_bits - (out_bits - 1))                    (Eq. 15)
 *   7. out_j = clamp(rshr_round(p_j * post.m, post.s) + post.zp, post.qmin, post.qmax)
 * Domain: variant in {0,1,2}; 16 <= i0 < 2^24 (< 2^16 for variant 2); n_shift >= 0 with (i0 << n_shift) < 2^24;
 * 2 <= out_bits <= 8; out_bits - 1 <= m_bits <= 31; cols * (i0 << n_shift) <= 2^m_bits
 * (else IPTQ_ERR_RANGE); 1 <= pre_m < 2^15; 0 <= pre_s <= 62.
 */
typedef struct {
    int32_t variant;
    int32_t i0;      /* floor(1 / S_delta) (Eq. 14) */
    int32_t n_shift; /* guard bits N; 0 is the literal Eq. 14 */
    int32_t m_bits;  /* M of Eq. 15 */
    int32_t out_bits; /* b of Eq. 15 */
    int32_t pre_m;
    int32_t pre_s;
    iptq_dyadic_t post;
    int32_t out_is_signed; /* 0: uint8_t output, 1: int8_t output */
    int32_t algo;          /* IPTQ_ALGO_* */
} iptq_softmax_params_t;

/*
 * Integer polynomial GELU of one value (Section 4.3, Eq. 3 and Eq. 5), p = 2 or 4:
 *   0. (int32 entry only) in = sat32(rshr_round(in * pre_m, pre_s)) unless (1, 0)
 *   1. q = clamp(in - zp_in, -max_abs_q, max_abs_q)
 *   2. t = min(|q|, -q_b) + q_b            in [q_b, 0]
 *   3. u = t^p + q_c                       (the square is reused for the quartic)
 *   4. v = (sign(q) * u + q_c) >> k        (1 + L on the scale where 1 is q_c / 2^k)
 *   5. w = q * v
 *   6. y = clamp(rshr_round(w * post.m, post.s) + post.zp, post.qmin, post.qmax)
 * Domain: q_b < 0 (|q_b| < 2^15 for p = 4, <= 2^30 for p = 2); q_c < 0; 0 <= k <= 62;
 * max_abs_q >= 1; ceil((|q_b|^p + 2|q_c|) / 2^k) * max_abs_q < 2^31 (so that q * v fits int32: a
 * negative numerator is floored away from zero) and |q_b|^p < 2^61, |q_c| < 2^60 (else
 * IPTQ_ERR_RANGE); for the int8 entry |zp_in| <= 128.
 */
typedef struct {
    int32_t variant;
    int32_t q_b;
    int64_t q_c;
    int32_t k;
    int32_t zp_in;
    int32_t max_abs_q;
    int32_t pre_m;
    int32_t pre_s;
    iptq_dyadic_t post; /* int8 output: qmin >= -128, qmax <= 127 */
    int32_t algo;       /* IPTQ_ALGO_AUTO: the polynomial is evaluated once per distinct centred
                           input into a per-workgroup table (int8 input: 256 entries; int32
                           input with max_abs_q <= 511: 2 max_abs_q + 1 entries) and gathered;
                           IPTQ_ALGO_GENERIC: polynomial per element */
} iptq_gelu_params_t;

/*
 * Which kernel family serves softmax rows of `cols` scores (16-byte aligned tensors, a call of
 * more than a few thousand rows).  *lanes: lanes that share a row; *blocks: 16-byte blocks (or
 * passes) per lane; both 0 where they do not apply.  Results never depend on the family.
 */
#define IPTQ_FAMILY_COMPILED 0          /* row length compiled in (197, 49, 198, 144, 257, 577) */
#define IPTQ_FAMILY_SLAB 1              /* slab kernel with a run-time row length */
#define IPTQ_FAMILY_WAVEFRONT_PER_ROW 2
#define IPTQ_FAMILY_WORKGROUP_PER_ROW 3
#define IPTQ_FAMILY_THREE_PASS 4        /* re-reads the row: any row length, slow */
int iptq_softmax_kernel_family(int32_t cols, int32_t *family, int32_t *lanes, int32_t *blocks);

/* Library version (major * 10000 + minor * 100 + patch). */
int iptq_version(void);

/* Static text for a return code. */
const char *iptq_strerror(int code);

/*
 * Requantization of an int32 tensor (the formula of iptq_dyadic_t).
 * d_in: n int32 (device, 4-byte aligned); d_out: n uint8_t (out_is_signed == 0) or int8_t
 * (== 1) (device); n >= 0 (0 is a successful no-op); p: host.  No further alignment is asked
 * of either pointer here or in the GELU entry points (fastest on the 16-byte grid, within 10 % of
 * that anywhere else).
 */
int iptq_requant(const int32_t *d_in, void *d_out, int64_t n, int32_t out_is_signed,
                 const iptq_dyadic_t *p, void *stream);

/*
 * Integer softmax over every row of a row-major [rows, cols] int32 score matrix
 * (Section 4.4, Eq. 6-15; steps listed at iptq_softmax_params_t).
 * d_scores: rows * cols int32 (device); d_bias: NULL or a row-major
 * [bias_period_rows, cols] int32 (device) added to row r from its row
 * (r mod bias_period_rows) - the Swin relative-position bias with
 * bias_period_rows = heads * window_tokens; d_out: rows * cols bytes (device), uint8_t or
 * int8_t per p->out_is_signed, must not overlap d_scores.
 * 0 <= rows < 2^31 (0 is a no-op), 1 <= cols <= IPTQ_COLS_MAX.
 * The post step runs at full speed when it is the identity, the int8 clip at 127, or the shift to
 * signed codes p - 128 (post = {1, 0, -128, -128, qmax >= 0}: the operand form of a signed 8-bit
 * matrix instruction for the product with V); any other post step goes through a small table.
 * Every shape gives the same bytes; speed depends on it.  Fastest: a row length of 197, 49, 198,
 * 144, 257 or 577; any other row length up to 40957 runs in the register-resident kernels with
 * a run-time row length, longer rows in a slower multi-pass kernel.  The tensors need their
 * natural alignment only (views into larger tensors run at the same speed as tensors on the
 * 16-byte grid); an additive table of any size is fused (a little faster when
 * bias_period_rows * cols is a multiple of 4, as with 4, 8, 16 or 32 Swin heads), except a
 * table with fewer rows than one wavefront's slab (64 rows divided by the lanes per row: 32 at
 * 49 columns, 8 or 16 at 197), or of 2^30 entries and more, which takes the three-pass kernel
 * (about a sixth of the speed).
 */
int iptq_softmax_i32(const int32_t *d_scores, const int32_t *d_bias, int64_t bias_period_rows,
                     void *d_out, int64_t rows, int32_t cols, const iptq_softmax_params_t *p,
                     void *stream);

/*
 * The same for windowed attention whose windows carry their own additive mask (the shifted-window
 * blocks of a Swin backbone; Section 4.1 keeps every operation of the block in integer
 * arithmetic): the rows of d_scores are ordered [image, window, head, query], each window has
 * `cols` queries and `cols` keys, and d_mask is a row-major [n_windows, cols, cols] int32 (device)
 * whose entry [w, q, k] is added to the score of key k in every row of window w, query q (0 or
 * INT32_MIN in a Swin model; any other value is an ordinary saturating addend).  Row r lies in
 * window (r div (heads * cols)) mod n_windows and is query r mod cols.  d_bias as above (normally
 * [heads * cols, cols] with bias_period_rows = heads * cols); either table may be NULL.  Nothing
 * is materialised: both tables are read beside the scores.  n_windows >= 1, heads >= 1,
 * n_windows * heads * cols < 2^31 (else IPTQ_ERR_SHAPE).
 * Speed: windows of 49 or 144 tokens with a bias run in the slab kernels (the extra table costs
 * about a sixth of the time; the packed form below costs almost nothing); any other shape, or a
 * mask without a bias, takes the slow three-pass kernel.
 */
int iptq_softmax_i32_windowed(const int32_t *d_scores, const int32_t *d_bias,
                              int64_t bias_period_rows, const int32_t *d_mask, int32_t n_windows,
                              int32_t heads, void *d_out, int64_t rows, int32_t cols,
                              const iptq_softmax_params_t *p, void *stream);

/*
 * The same with the mask handed over one bit per key, for masks whose entries are 0 or INT32_MIN
 * only (a Swin model's are): d_mask_bits is a [n_windows, cols, ceil(cols / 64)] array of 64-bit
 * words (device, 8-byte aligned); bit (k mod 64) of word (k div 64) of row [w, q] set means key k
 * is masked for query q of window w; bits beyond `cols` are ignored.  Identical results to
 * iptq_softmax_i32_windowed with the int32 mask those bits stand for; the mask then costs one
 * 8-byte load per row and two instructions per score instead of a third table read beside the
 * scores (Swin-B stage 1 at batch 64: 35 us against 34 us without a mask and 40 us with the int32
 * mask).
 * Speed: windows of 49 or 144 tokens with a bias run in the slab kernels; any other shape takes
 * the slow three-pass kernel.  Errors as for iptq_softmax_i32_windowed; IPTQ_ERR_ALIGN if
 * d_mask_bits is not 8-byte aligned; a batched problem that carries both forms of the mask is
 * refused with IPTQ_ERR_PARAM.
 */
int iptq_softmax_i32_windowed_bits(const int32_t *d_scores, const int32_t *d_bias,
                                   int64_t bias_period_rows, const uint64_t *d_mask_bits,
                                   int32_t n_windows, int32_t heads, void *d_out, int64_t rows,
                                   int32_t cols, const iptq_softmax_params_t *p, void *stream);

/*
 * Packs a [n_windows, cols, cols] int32 mask (device) into that form: a bit is set where the
 * entry equals INT32_MIN, any other entry counts as "not masked".  d_mask_bits:
 * n_windows * cols * ceil(cols / 64) words (device, 8-byte aligned, caller-owned, must not
 * overlap d_mask).  Done once per model, when the masks are built.  n_windows >= 0 (0: no-op).
 */
int iptq_pack_window_mask(const int32_t *d_mask, int32_t n_windows, int32_t cols,
                          uint64_t *d_mask_bits, void *stream);

/*
 * Integer GELU (Section 4.3, Eq. 3 and 5; steps listed at iptq_gelu_params_t) of n int8
 * activations.  d_out may equal d_in (in place); partial overlap is not allowed.
 */
int iptq_gelu_i8(const int8_t *d_in, int8_t *d_out, int64_t n, const iptq_gelu_params_t *p,
                 void *stream);

/* Same on int32 accumulators with the requantization (pre_m, pre_s) fused in front. */
int iptq_gelu_i32(const int32_t *d_in, int8_t *d_out, int64_t n, const iptq_gelu_params_t *p,
                  void *stream);

/*
 * Batched forms: several independent problems in as few kernel launches as possible (at most
 * IPTQ_BATCH_MAX problems per call), e.g. the layers of a model sweep or the stages of a Swin
 * backbone.  Results are identical to one single call per problem; all problems are checked
 * before anything is enqueued.  The per-layer variant choice of Section 4.2 is the `variant`
 * field of each problem's parameters.  Softmax problems of one call share the row length.
 */
#define IPTQ_BATCH_MAX 16

typedef struct {
    const int32_t *d_scores;  /* rows * cols int32 (device) */
    const int32_t *d_bias;    /* NULL or [bias_period_rows, cols] int32 (device) */
    int64_t bias_period_rows;
    void *d_out;              /* rows * cols bytes (device) */
    int64_t rows;
    iptq_softmax_params_t params;
    const int32_t *d_mask;    /* NULL or the per-window mask of iptq_softmax_i32_windowed */
    int32_t n_windows;
    int32_t heads;
    const uint64_t *d_mask_bits; /* NULL or the mask one bit per key (iptq_softmax_i32_windowed_bits);
                                    at most one of d_mask and d_mask_bits */
} iptq_softmax_problem_t;

typedef struct {
    const int8_t *d_in; /* n int8 (device) */
    int8_t *d_out;      /* n int8 (device), may equal d_in */
    int64_t n;
    iptq_gelu_params_t params;
} iptq_gelu_problem_t;

int iptq_softmax_i32_batch(const iptq_softmax_problem_t *problems /*host*/, int32_t n_problems,
                           int32_t cols, void *stream);
int iptq_gelu_i8_batch(const iptq_gelu_problem_t *problems /*host*/, int32_t n_problems,
                       void *stream);

/*
 * Layer-strided forms of the same: layer l reads d_scores + l * in_stride (elements) and
 * writes d_out + l * out_stride (bytes) with p[l]; all layers share rows and cols (or n);
 * any number of layers.  No bias.
 */
int iptq_softmax_i32_layers(const int32_t *d_scores, int64_t in_stride, void *d_out,
                            int64_t out_stride, int64_t rows, int32_t cols, int32_t n_layers,
                            const iptq_softmax_params_t *p, void *stream);
int iptq_gelu_i8_layers(const int8_t *d_in, int64_t in_stride, int8_t *d_out, int64_t out_stride,
                        int64_t n, int32_t n_layers, const iptq_gelu_params_t *p, void *stream);

/*
 * Host-only helpers: real scales -> integer constants, once, before inference (the
 * polynomial coefficients of Section 4.3 become integer constants; floor(1/S), Eq. 14).
 * IEEE double.
 */

/* ratio ~ m / 2^s with |m| in [2^14, 2^15) and the largest s <= 62 (see the .cpp for ties). */
int iptq_make_dyadic(double ratio, int32_t *m, int32_t *s);

/* i0 = floor(1/s_delta); n_shift = max(0, 15 - bitlen(i0)) lowered until
 * cols * (i0 << n_shift) <= 2^30; m_bits = 30; out_bits = 8; identity pre/post
 * (int8 output clips the code 128 to 127). */
int iptq_softmax_prepare(double s_delta, int32_t cols, int32_t variant, int32_t out_is_signed,
                         iptq_softmax_params_t *out);

/* S_e = s_in / sqrt 2; q_b = floor(b / S_e); q_c = floor(1 / (a S_e^p));
 * k = smallest shift keeping q * v inside int32 for |q| <= max_abs_q;
 * post = dyadic(s_in * a * S_e^p * 2^k / 2 / s_out), zero-point zp_out, int8 clip. */
int iptq_gelu_prepare(double s_in, double s_out, int32_t zp_in, int32_t zp_out, int32_t variant,
                      int32_t max_abs_q, iptq_gelu_params_t *out);

/*
 * Host-only: the Unified Metric that picks the approximation function of each activation layer
 * (Section 4.5, Eq. 16-20), i.e. the `variant` field of the parameter structs.  For one layer
 * and one candidate, from the layer's real-valued output x[0..n) and the candidate's dequantized
 * output x_hat[0..n) (both host, double):
 *   q_db  = 10 log10(mean x^2 / mean (x - x_hat)^2)   quantization sensitivity, SQNR in dB (Eq. 18;
 *           the factor follows the section's worked example: power 10^4 against error powers 100
 *           and 60 gives 20 dB and 22.21 dB)
 *   p     = sum (x - x_hat)^2                           quantization perturbation (Eq. 19)
 *   c     = op_count                                    integer operations of the layer (Eq. 20)
 *   n_*   = log(1 + exp(.)) of each                     Softplus (Eq. 17)
 *   score = 3 / (1 / n_q + n_p + n_c)                   one term of Eq. 16
 * The candidate with the highest score is assigned to the layer (iptq_unified_select: the first
 * among equals), and the metric Omega of a model is the sum of its layers' assigned scores.
 * mode IPTQ_METRIC_LITERAL takes p and c as above; with whole-layer values they are 10^3..10^9,
 * n_p + n_c = p + c swamps 1 / n_q, and the cheapest candidate always wins.  The normalisation
 * the paper uses is not printed; IPTQ_METRIC_PER_ELEMENT divides p and c by n.
 * iptq_softmax_op_count / iptq_gelu_op_count: the library's count of arithmetic and bit
 * operations of the steps listed at the parameter structs (softmax: 18, 22, 25 per score for
 * variants 0, 1, 2 plus one division per row; GELU: 17, 18 per value); -1 on a bad argument.
 */
#define IPTQ_METRIC_LITERAL 0
#define IPTQ_METRIC_PER_ELEMENT 1
typedef struct {
    double q_db, p, c;
    double n_q, n_p, n_c;
    double score;
} iptq_metric_t;
int iptq_unified_metric(const double *x, const double *x_hat, int64_t n, double op_count,
                        int32_t mode, iptq_metric_t *out);
int iptq_unified_select(const iptq_metric_t *candidates, int32_t n_candidates, int32_t *best);
int64_t iptq_softmax_op_count(int32_t variant, int64_t rows, int32_t cols);
int64_t iptq_gelu_op_count(int32_t variant, int64_t n);

#ifdef __cplusplus
}
#endif
#endif /* IPTQ_H */
