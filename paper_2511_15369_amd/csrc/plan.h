// Host-side plans: validated call parameters turned into the integer constants the
// kernels take by value.  Everything here is plain C++ (no HIP types) so that the checks
// can be exercised without a GPU.
#pragma once

#include <stdint.h>

#include "../../include/iptq.h"

namespace iptq {

// Constants of one softmax launch (Section 4.4).  All derived on the host.
struct SoftmaxDev {
    int32_t i0;         // floor(1 / S_delta)
    int32_t i0n;        // i0 << N: the integer image of 1.0
    int32_t n_shift;    // N
    uint32_t magic;     // q = mulhi(n, magic) >> magic_sh == n div i0 for 0 <= n <= n_max
    int32_t magic_sh;
    int32_t d_clamp;    // D: deltas below -D have Qexp == 0 and are clamped to -D
    int32_t mode16;     // 0: 32-bit lanes only; 1: packed 16-bit path valid; 2: same with n << t16
    uint32_t mg24;      // packed path divider: q = bits 47..32 of (n << t16) * mg24
    int32_t t16;
    int32_t m_bits;     // M
    int32_t p_shift;    // M - (b - 1)
    int32_t pre_m, pre_s;
    // pre-requantization without a 64-bit shift (pre_mode 1, pre_s >= 16): the result is
    // ((x * pre_mul + pre_rnd) >> 32) >> pre_sh2.  pre_mode 0: none, 2: general form only.
    int32_t pre_mode;
    int32_t pre_mul;
    int32_t pre_sh2;
    int64_t pre_rnd;
    // pre-requantization folded into Eq. 6 (pre_rowconst 1; pre_s in [16, 31], packed path only):
    // with d = max - x >= 0 on the raw scores, r(x) - r(max) == -((d * pre_m + c) >> pre_s), c a
    // constant of the row (2^s - 1 - ((max * pre_m + 2^(s-1)) mod 2^s)); d is clamped at pre_dmax =
    // ceil(D 2^s / pre_m), beyond which the exponential is 0 anyway, so the product fits 32 bits.
    int32_t pre_rowconst;
    uint32_t pre_dmax;
    int32_t post_m, post_s, post_zp, qmin, qmax;
    // The post step "minus 128, no clip inside [-128, 0]" (signed int8 probabilities around a
    // zero-point of -128, the operand form of a signed 8-bit matrix instruction): on bytes that
    // are at most 128 it is one exclusive-or.  0x80808080 then, else 0.
    uint32_t post_xor;
    int32_t variant;
    // second-degree form (variant 2): floor(y^2 / (2 i0)) == mulhi(y^2, d2_magic) >> d2_sh for y^2 < 2^31
    uint32_t d2_magic;
    int32_t d2_sh;
    // bias addressing: row index modulo the period by multiply-high
    int32_t bias_period_rows;
    uint32_t period_magic;
    int32_t period_sh;
    // per-window mask [n_windows, cols, cols] (0: none): rows are ordered [image, window, head,
    // query]; row r lies in window (r mod mask_period_rows) div group_rows and is query
    // (r mod group_rows) mod cols of it.  group_rows = heads * cols, mask_period_rows =
    // n_windows * group_rows; both divisions by multiply-high.
    int32_t n_windows;
    int32_t group_rows;
    int32_t mask_period_rows;
    uint32_t mperiod_magic, group_magic;
    int32_t mperiod_sh, group_sh;
};

// Constants of one GELU launch (Section 4.3).
struct GeluDev {
    int32_t quartic;    // 1: p = 4, 0: p = 2
    int32_t q_b;
    int64_t q_c;
    int32_t k;
    int32_t zp_in;
    int32_t max_abs_q;
    int32_t pre_m, pre_s;
    int32_t post_m, post_s, post_zp, qmin, qmax;
    int32_t fast;       // 1: t^2 fits 32 bits and post_s >= 16, the short evaluation applies
    int32_t pre_mode;   // 0: no pre-requantization, 1: pre_s >= 15 (result fits 32 bits), 2: general
};

struct DyadicDev {
    int32_t m, s, zp, qmin, qmax;
};

// Unsigned division by a constant through multiply-high: for every 0 <= n < 2^nbits,
// (mulhi32(n, magic) >> sh) == n / d.  Requires 1 <= d < 2^nbits and nbits <= 31.
// Returns false if no 32-bit magic exists for that range (cannot happen for nbits <= 31).
bool make_magic_u32(uint32_t d, int nbits, uint32_t *magic, int32_t *sh);

// n(d) = -Qp for delta = -d: d + ceil(d/2) - ceil(d/16) (Eq. 7 with floor shifts).
int64_t neg_qp_of(int64_t d);

int check_dyadic(const iptq_dyadic_t *p, int out_is_signed);
int plan_requant(const iptq_dyadic_t *p, int out_is_signed, DyadicDev *out);
int plan_softmax(const iptq_softmax_params_t *p, int64_t rows, int32_t cols, int has_bias,
                 int64_t bias_period_rows, SoftmaxDev *out);
// Adds the per-window mask's addressing constants to a plan made by plan_softmax.
int plan_softmax_mask(int64_t n_windows, int64_t heads, int32_t cols, SoftmaxDev *out);
int plan_gelu(const iptq_gelu_params_t *p, int is_i8_entry, GeluDev *out);

}  // namespace iptq
