// Fixed-row-length integer softmax kernel for gfx950 (Section 4.4, Eq. 6-15).
//
// A wavefront owns 64/K whole rows (a "slab"), K lanes per row.  The slab is contiguous
// and a whole number of 16-byte chunks in both the int32 input and the byte output, so all
// global traffic is full dwordx4 (at the tensor's own alignment: a view into a larger tensor
// need not sit on the 16-byte grid): the slab is copied flat into LDS (with the additive
// bias fused into the copy), lanes then read their rows from LDS on the 16-byte grid of the
// slab ("blocks" of 4 elements; a row that does not start on that grid ignores the
// neighbours' elements in its first and last block), results are assembled as bytes in
// LDS and stored flat.  Only wavefront-level ordering is needed: no workgroup barrier.
//
// Two arithmetic paths give identical results:
//   MODE 0  every step in 32-bit lanes; valid for the whole parameter domain.
//   MODE 1  two elements per 32-bit lane in packed 16-bit (v_pk_*), for the usual case
//           where the clamped delta, n = -Qp and (i0 << N) all fit 16 bits.
//   MODE 2  as MODE 1, with n pre-shifted so that the divider's multiplier fits 24 bits
//           for small i0.
#pragma once

#include <hip/hip_runtime.h>

#include <type_traits>

#include "device_common.h"
#include "plan.h"

namespace iptq {

typedef short s16x2 __attribute__((ext_vector_type(2)));
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));

enum { PM_NONE = 0, PM_CLAMP127 = 1, PM_GENERAL = 2 };

// One launch serves up to kBatchMax independent problems of the same row length (the layers
// of a model sweep, the stages of a Swin backbone): workgroups [first_wg, next first_wg)
// belong to item i.  The table travels in the kernel arguments.
constexpr int kBatchMax = 16;
// wavefronts per workgroup of the row kernel; they do not cooperate, so this only sets the
// granularity at which the dispatcher hands out work and LDS
constexpr int kRowsWpb = 4;
struct SoftmaxItem {
    const int32_t *scores;
    const int32_t *bias;
    const int32_t *mask;  // per-window mask [n_windows, cols, cols] or nullptr
    const uint64_t *mask_bits;   // the same mask one bit per key, [n_windows, cols, ceil(cols / 64)] words, or nullptr
    uint8_t *out;
    int64_t n_slabs;      // the last one may be partial
    uint32_t first_wg;
    int32_t tail_rows;    // rows of the last slab if it is partial, else 0
    // Slabs whose first rows are congruent modulo the bias period read the same rows of the
    // additive table.  share_q = period / gcd(period, rows per slab) is the distance, in slabs,
    // between two such slabs; with share_q != 0 the wavefronts of a workgroup take slabs
    // share_q apart (workgroup w, wavefront v: slab (w / q) * WPB * q + v * q + w % q), so that
    // the table rows reach the compute unit's L1 once per workgroup instead of once per
    // wavefront.  0: consecutive slabs.
    uint32_t share_q, share_magic;
    int32_t share_sh;     // w / share_q == mulhi(w, share_magic) >> share_sh
    SoftmaxDev P;
};
struct SoftmaxBatch {
    int32_t n_items;
    SoftmaxItem item[kBatchMax];
};
static_assert(sizeof(SoftmaxBatch) <= 4096, "kernel arguments are limited to 4 KiB");

// rshr_round(x * pre_m, pre_s) for pre_s >= 16 (SoftmaxDev::pre_mode 1): one 64-bit
// multiply-add and a 32-bit shift of its high half.
IPTQ_DEV int32_t pre_requant_narrow(int32_t x, int32_t pre_mul, int64_t pre_rnd, int32_t pre_sh2)
{
    const int64_t t = (int64_t)x * (int64_t)pre_mul + pre_rnd;
    return (int32_t)(t >> 32) >> pre_sh2;
}

// One exponential in 32-bit lanes (Eq. 7-10 / 13-14).  x is the (biased) score, `lower`
// is max(row) - D saturated, mx the row maximum.  Elements at or below `lower` get the
// same all-zero result as their true value, which keeps every intermediate in 32 bits.
template <int VARIANT, bool EXPLICIT_MASK>
IPTQ_DEV uint32_t bit_exp_dev(int32_t x, int32_t lower, int32_t mx, const SoftmaxDev &P)
{
    const int32_t xc = max(x, lower);
    const int32_t dl = xc - mx;                        // Eq. 6, in [-D, 0]
    const int32_t s1 = dl >> 1, s4 = dl >> 4;
    const int32_t n = (s4 - dl) - s1;                  // -Qp of Eq. 7, >= 0
    const uint32_t q = mulhi_u32((uint32_t)n, P.magic) >> P.magic_sh;   // Eq. 8: n div i0
    const int32_t nr = (int32_t)__umul24(q, (uint32_t)P.i0) - n;        // -r in (-i0, 0]
    int32_t fr = nr >> 1;                              // Eq. 10: x / 2
    if (VARIANT >= 1) fr += (nr >> 3) + (nr >> 4);     // Eq. 13: (0.1011)b x
    if (VARIANT == 2)                                  // Eq. 11 with D = 2: + floor(y^2 / (2 i0))
        fr += (int32_t)(mulhi_u32((uint32_t)(fr * fr), P.d2_magic) >> P.d2_sh);
    const uint32_t base = ((uint32_t)fr << P.n_shift) + (uint32_t)P.i0n;  // Eq. 14, << N
    uint32_t e = base >> q;                            // Eq. 9 (q <= 31 by the clamp)
    if (EXPLICIT_MASK) e = (x == kI32Min) ? 0u : e;
    return e;
}

template <int POSTMODE>
IPTQ_DEV uint32_t post_dev(uint32_t p, const SoftmaxDev &P)
{
    if (POSTMODE == PM_NONE) return p;
    if (POSTMODE == PM_CLAMP127) return min(p, 127u);
    // general dyadic requantization; p <= 2^(b-1) so 64-bit arithmetic is ample
    const int64_t rnd = P.post_s > 0 ? ((int64_t)1 << (P.post_s - 1)) : 0;
    int64_t v = (((int64_t)p * P.post_m + rnd) >> P.post_s) + P.post_zp;
    v = v < P.qmin ? P.qmin : v;
    v = v > P.qmax ? P.qmax : v;
    return (uint32_t)(int32_t)v & 0xffu;
}

// row index modulo the bias period without a divide
IPTQ_DEV uint32_t row_mod_period(uint32_t row, const SoftmaxDev &P)
{
    if (P.bias_period_rows == 1) return 0u;
    const uint32_t q = mulhi_u32(row, P.period_magic) >> P.period_sh;
    return row - q * (uint32_t)P.bias_period_rows;
}

// Four consecutive entries of the additive table from entry o (0 <= o < pe entries in all),
// continuing at entry 0 past the table's end.  The table's size need not be a multiple of
// four (Swin with 3 or 6 heads: 147 * 49 entries): the load is placed so that it ends inside
// the table (`a`), and a chunk that straddles the end takes its last entries from `first4`
// (entries 0..3, loaded once per wavefront).  Branch-free; `sh` is 0 for every other chunk.
IPTQ_DEV i32x4 bias_chunk_wrapping(const int32_t *bias, uint32_t o, uint32_t pe, const i32x4 first4)
{
    const uint32_t a = min(o, pe - 4u);
    const uint32_t sh = o - a;
    const i32x4 A = load_i32x4(bias + a);
    i32x4 r;
    r.x = sh == 0 ? A.x : (sh == 1 ? A.y : (sh == 2 ? A.z : A.w));
    r.y = sh == 0 ? A.y : (sh == 1 ? A.z : (sh == 2 ? A.w : first4.x));
    r.z = sh == 0 ? A.z : (sh == 1 ? A.w : (sh == 2 ? first4.x : first4.y));
    r.w = sh == 0 ? A.w : (sh == 1 ? first4.x : (sh == 2 ? first4.y : first4.z));
    return r;
}

// Where the rows of a slab find their rows of the per-window mask.  Consecutive score rows are
// consecutive mask rows until the query index wraps (every `cols` rows: the next head of the
// same window starts over at the window's first mask row, the next window at its own), and a slab
// has fewer rows than a window has queries, so a slab's mask entries are at most two contiguous
// runs: slab elements [0, e1) take mask[off1 + e], the rest mask[off2 + (e - e1)].  If e1 is not
// a multiple of four, one 16-byte chunk (slab elements o_s .. o_s+3) holds entries of both runs;
// its four entries are put together once per wavefront (`straddle`), every other chunk is one load.
struct MaskRuns {
    uint32_t off1, off2;  // element offsets into the mask
    uint32_t e1;          // a multiple of cols; at least the slab size when there is no second run
    uint32_t o_s;         // first slab element of the chunk that straddles, or 0xffffffff
    i32x4 straddle;
};
template <int COLS, int RPW>
IPTQ_DEV MaskRuns mask_runs_of_slab(const int32_t *mask, uint32_t row0, const SoftmaxDev &P)
{
    uint32_t rm = 0;                                  // row modulo the mask period
    if (P.mask_period_rows >= 2)
        rm = row0 - (mulhi_u32(row0, P.mperiod_magic) >> P.mperiod_sh) * (uint32_t)P.mask_period_rows;
    const uint32_t w1 = P.group_rows >= 2 ? mulhi_u32(rm, P.group_magic) >> P.group_sh : rm;   // window of row0
    const uint32_t rin = rm - w1 * (uint32_t)P.group_rows;       // row inside [head, query] of that window
    const uint32_t q0 = rin % (uint32_t)COLS;                    // compile-time divisor: a multiply-high
    const uint32_t rd = (uint32_t)COLS - q0;                     // rows until the query index wraps
    uint32_t w2 = w1;
    if (rin + rd >= (uint32_t)P.group_rows) w2 = (w1 + 1 == (uint32_t)P.n_windows) ? 0u : w1 + 1;
    MaskRuns R;
    R.off1 = (w1 * (uint32_t)COLS + q0) * (uint32_t)COLS;
    R.off2 = w2 * (uint32_t)(COLS * COLS);
    R.e1 = rd * (uint32_t)COLS;
    R.o_s = 0xffffffffu;
    R.straddle = (i32x4){0, 0, 0, 0};
    const uint32_t c1 = R.e1 & 3u;                    // entries of the straddling chunk in the first run
    if (R.e1 < (uint32_t)(RPW * COLS) && c1 != 0) {
        R.o_s = R.e1 - c1;
        const i32x4 A = load_i32x4(mask + R.off1 + R.e1 - 4u);    // the first run's last four entries
        const i32x4 F = load_i32x4(mask + R.off2);                // the second run's first four
        R.straddle.x = c1 == 1 ? A.w : (c1 == 2 ? A.z : A.y);
        R.straddle.y = c1 == 1 ? F.x : (c1 == 2 ? A.w : A.z);
        R.straddle.z = c1 == 1 ? F.y : (c1 == 2 ? F.x : A.w);
        R.straddle.w = c1 == 1 ? F.z : (c1 == 2 ? F.y : F.x);
    }
    return R;
}

// Mask entries of the chunk that starts at slab element o.  Branch-free: the load of the
// straddling chunk is placed inside the first run and its result replaced.
IPTQ_DEV i32x4 mask_chunk(const int32_t *mask, const MaskRuns &R, uint32_t o)
{
    // (a bit select, not `?:`: the compiler turned the conditional into a lane-divergent branch,
    // which cut the copy loop into blocks and left one pass of loads in flight at a time)
    const uint32_t in2 = 0u - (uint32_t)(o >= R.e1);
    const uint32_t off = ((R.off2 + (o - R.e1)) & in2) | ((R.off1 + min(o, R.e1 - 4u)) & ~in2);
    i32x4 m = load_i32x4(mask + off);
    const bool st = o == R.o_s;
    m.x = st ? R.straddle.x : m.x;
    m.y = st ? R.straddle.y : m.y;
    m.z = st ? R.straddle.z : m.z;
    m.w = st ? R.straddle.w : m.w;
    return m;
}

// score + bias + mask entries with "minus infinity if any is": one test for the three
IPTQ_DEV int32_t add_two_table_entries(int32_t x, int32_t b, int32_t m)
{
    const int32_t s = sat_add_i32(sat_add_i32(x, b), m);
    return min(min(x, b), m) == kI32Min ? kI32Min : s;
}

// bytes 3 of (a, b, c, d) -> one dword (a in byte 0)
IPTQ_DEV uint32_t pack_top_bytes(uint32_t a, uint32_t b, uint32_t c, uint32_t d)
{
    const uint32_t ab = __builtin_amdgcn_perm(b, a, 0x0c0c0703u);
    const uint32_t cd = __builtin_amdgcn_perm(d, c, 0x0c0c0703u);
    return __builtin_amdgcn_perm(cd, ab, 0x05040100u);
}

// per-byte min(v, 127) for bytes that are at most 128
IPTQ_DEV uint32_t clamp127_bytes(uint32_t w) { return w - ((w >> 7) & 0x01010101u); }

// The general post step through a table: a probability has at most 2^(b-1) + 1 <= 129
// values, so a wavefront evaluates the dyadic requantization once per value into LDS
// (kPostLutBytes per wavefront) and every output byte is one gather.
constexpr int kPostLutBytes = 144;
IPTQ_DEV uint32_t post_lut_gather(const uint8_t *lut, uint32_t w)
{
    const uint32_t y0 = lut[w & 0xffu], y1 = lut[(w >> 8) & 0xffu];
    const uint32_t y2 = lut[(w >> 16) & 0xffu], y3 = lut[w >> 24];
    return y0 | (y1 << 8) | (y2 << 16) | (y3 << 24);
}

// Eq. 15 for one block of four exponentials in 32-bit lanes -> four output bytes
template <int POSTMODE>
IPTQ_DEV uint32_t normalise4(uint32_t e0, uint32_t e1, uint32_t e2, uint32_t e3, uint32_t f,
                             uint32_t f_top, const SoftmaxDev &P)
{
    if (POSTMODE != PM_GENERAL && P.p_shift <= 24) {
        // (f << (24 - p_shift)) * Qexp <= 2^31 carries p in its top byte
        uint32_t w = pack_top_bytes(e0 * f_top, e1 * f_top, e2 * f_top, e3 * f_top);
        if (POSTMODE == PM_CLAMP127) w = clamp127_bytes(w);
        return w;
    }
    const uint32_t p0 = post_dev<POSTMODE>((e0 * f) >> P.p_shift, P);
    const uint32_t p1 = post_dev<POSTMODE>((e1 * f) >> P.p_shift, P);
    const uint32_t p2 = post_dev<POSTMODE>((e2 * f) >> P.p_shift, P);
    const uint32_t p3 = post_dev<POSTMODE>((e3 * f) >> P.p_shift, P);
    return p0 | (p1 << 8) | (p2 << 16) | (p3 << 24);
}

IPTQ_DEV uint32_t mulhi_u24(uint32_t a, uint32_t b)   // both below 2^24: bits 47..32 of a*b
{
    return (uint32_t)(((uint64_t)(a & 0xffffffu) * (uint64_t)(b & 0xffffffu)) >> 32);
}

// Two exponentials at once in packed 16-bit lanes.  Preconditions (checked on the host,
// SoftmaxDev::p16): D <= 32767, n_max <= 65535 >> t16, i0 << N < 2^15 (so q <= 15 at the
// clamp), divider multiplier mg24 < 2^24 exact for (n << t16).
// From the two stabilised scores of Eq. 6 (any value in [-32768, 0]) on.
// N = 2: one pair; N = 4: the two pairs of a 16-byte block side by side, every packed step as two
// independent instructions back to back (a single pair is one dependent chain, which leaves the
// vector unit waiting on itself when few wavefronts share it, as at the end of a launch).
template <int N> struct Packed16;
template <> struct Packed16<2> {
    typedef s16x2 S;
    typedef u16x2 U;
    typedef uint32_t W __attribute__((ext_vector_type(1)));    // the same bits as 32-bit words
};
template <> struct Packed16<4> {
    typedef short S __attribute__((ext_vector_type(4)));
    typedef unsigned short U __attribute__((ext_vector_type(4)));
    typedef uint32_t W __attribute__((ext_vector_type(2)));
};

template <int VARIANT, bool SHIFTED, int N>
IPTQ_DEV typename Packed16<N>::U bit_exp_of_deltas(typename Packed16<N>::S dl, const SoftmaxDev &P)
{
    typedef typename Packed16<N>::S S;
    typedef typename Packed16<N>::U U;
    const short nd = (short)(-P.d_clamp);
    dl = __builtin_elementwise_max(dl, (S)nd);                 // Eq. 6 with the clamp at -D
    const S s1 = dl >> 1, s4 = dl >> 4;
    const U n = (U)((s4 - dl) - s1);                           // -Qp of Eq. 7
    U ns = n;
    if (SHIFTED) ns = n << (unsigned short)P.t16;
    U q;
#pragma unroll
    for (int i = 0; i < N / 2; ++i) {                          // Eq. 8: n div i0, per 32-bit word of the vector
        const uint32_t nw = __builtin_bit_cast(typename Packed16<N>::W, ns)[i];
        q[2 * i] = (unsigned short)mulhi_u24(nw & 0xffffu, P.mg24);
        // (a field extract folds into the multiply's operand select)
        q[2 * i + 1] = (unsigned short)mulhi_u24(__builtin_amdgcn_ubfe(nw, 16, 16), P.mg24);
    }
    const unsigned short i0 = (unsigned short)P.i0;
    const S nr = (S)(q * (U)i0 - n);                           // -r in (-i0, 0]
    S fr = nr >> 1;                                            // Eq. 10
    if (VARIANT >= 1) fr = fr + (nr >> 3) + (nr >> 4);         // Eq. 13
    if (VARIANT == 2) {
        // Eq. 11 with D = 2: + floor(y^2 / (2 i0)).  |y| < 0.6875 i0 < 2^15, so the square needs a
        // 32-bit lane per element (24-bit multiply, multiply-high by the reciprocal of 2 i0); the
        // quotient is below i0 / 4 and goes back into the packed vector.
        S t;
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int32_t y = fr[i];
            t[i] = (short)(mulhi_u32((uint32_t)__mul24(y, y), P.d2_magic) >> P.d2_sh);
        }
        fr = fr + t;
    }
    const unsigned short sc = (unsigned short)(1u << P.n_shift), one = (unsigned short)P.i0n;
    const U base = (U)fr * (U)sc + (U)one;                     // Eq. 14, << N
    return base >> q;                                          // Eq. 9 (q <= 15)
}

template <int VARIANT, bool SHIFTED>
IPTQ_DEV u16x2 bit_exp_pair_of_deltas(s16x2 dl, const SoftmaxDev &P)
{
    return bit_exp_of_deltas<VARIANT, SHIFTED, 2>(dl, P);
}

template <int VARIANT, bool SHIFTED>
IPTQ_DEV u16x2 bit_exp_pair(int32_t xa, int32_t xb, int32_t mx, const SoftmaxDev &P)
{
    const int32_t da = __builtin_elementwise_sub_sat(xa, mx);
    const int32_t db = __builtin_elementwise_sub_sat(xb, mx);
    return bit_exp_pair_of_deltas<VARIANT, SHIFTED>(__builtin_amdgcn_cvt_pk_i16(da, db), P);   // saturating pack
}

// The four scores of a 16-byte block -> their exponentials as two packed words.
template <int VARIANT, bool SHIFTED>
IPTQ_DEV void bit_exp_block(const int32_t (&x)[4], int32_t mx, const SoftmaxDev &P, uint32_t (&e)[2])
{
    const s16x2 lo = __builtin_amdgcn_cvt_pk_i16(__builtin_elementwise_sub_sat(x[0], mx),
                                                 __builtin_elementwise_sub_sat(x[1], mx));
    const s16x2 hi = __builtin_amdgcn_cvt_pk_i16(__builtin_elementwise_sub_sat(x[2], mx),
                                                 __builtin_elementwise_sub_sat(x[3], mx));
    const Packed16<4>::U q = bit_exp_of_deltas<VARIANT, SHIFTED, 4>(__builtin_shufflevector(lo, hi, 0, 1, 2, 3), P);
    e[0] = __builtin_bit_cast(uint32_t, __builtin_shufflevector(q, q, 0, 1));
    e[1] = __builtin_bit_cast(uint32_t, __builtin_shufflevector(q, q, 2, 3));
}

// The same with the requantization of the scores folded in (SoftmaxDev::pre_rowconst): the scores
// and mx are raw, c_row is the row's constant.
template <int VARIANT, bool SHIFTED>
IPTQ_DEV void bit_exp_block_requant(const int32_t (&x)[4], int32_t mx, uint32_t c_row, const SoftmaxDev &P,
                                    uint32_t (&e)[2])
{
    Packed16<4>::S d;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t dd = min((uint32_t)mx - (uint32_t)x[i], P.pre_dmax);     // mx >= x: exact as unsigned
        d[i] = (short)((__umul24(dd, (uint32_t)P.pre_m) + c_row) >> P.pre_s);    // r(mx) - r(x), at most D + 1
    }
    const Packed16<4>::U q = bit_exp_of_deltas<VARIANT, SHIFTED, 4>((Packed16<4>::S)0 - d, P);
    e[0] = __builtin_bit_cast(uint32_t, __builtin_shufflevector(q, q, 0, 1));
    e[1] = __builtin_bit_cast(uint32_t, __builtin_shufflevector(q, q, 2, 3));
}

// The arithmetic of one wavefront's slab once its rows sit in registers: exponentials, row
// sum, reciprocal, probabilities -> four output bytes per block in w[].
// Row sum over the K lanes that share a row (the default reducer of softmax_slab_math).
template <int K>
struct LaneGroupSum {
    IPTQ_DEV uint32_t operator()(uint32_t v) const { return group_sum_u32<K>(v); }
};

// SUM: how the per-lane partial sums of a row are combined.
// PRE: x and mx are raw scores and the requantization in front is folded into the exponentials
// (packed path only; the caller has checked SoftmaxDev::pre_rowconst and that no row is "low").
template <int K, int SLOTS, int MODE, int VARIANT, int POSTMODE, class SUM = LaneGroupSum<K>, bool PRE = false>
IPTQ_DEV void softmax_slab_math(int32_t (&x)[SLOTS][4], uint32_t (&w)[SLOTS], int32_t mx,
                                int32_t lower, bool any_low, const uint8_t *lut, const SoftmaxDev &P,
                                const SUM &row_sum = SUM(), uint32_t c_row = 0)
{
    if (MODE != 0 && __builtin_expect(!any_low, 1)) {
        // ---- packed 16-bit path
        uint32_t e2[SLOTS][2];
        uint32_t sum = 0;
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            if (PRE) bit_exp_block_requant<VARIANT, MODE == 2>(x[s], mx, c_row, P, e2[s]);
            else bit_exp_block<VARIANT, MODE == 2>(x[s], mx, P, e2[s]);
            sum = __builtin_amdgcn_udot2(__builtin_bit_cast(u16x2, e2[s][0]), (u16x2){1, 1}, sum, false);
            sum = __builtin_amdgcn_udot2(__builtin_bit_cast(u16x2, e2[s][1]), (u16x2){1, 1}, sum, false);
        }
        sum = row_sum(sum);
        const uint32_t f_top = floor_pow2_div(P.m_bits, sum) << (24 - P.p_shift);   // < 2^24
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            const uint32_t a = __umul24(e2[s][0] & 0xffffu, f_top), b = __umul24(e2[s][0] >> 16, f_top);
            const uint32_t c = __umul24(e2[s][1] & 0xffffu, f_top), d = __umul24(e2[s][1] >> 16, f_top);
            uint32_t ww = pack_top_bytes(a, b, c, d);
            if (POSTMODE == PM_CLAMP127) ww = clamp127_bytes(ww);
            if (POSTMODE == PM_GENERAL) ww = post_lut_gather(lut, ww);
            w[s] = ww;
        }
    } else {
        // ---- 32-bit path
        uint32_t sum = 0;
        if (__builtin_expect(!any_low, 1)) {
#pragma unroll
            for (int s = 0; s < SLOTS; ++s)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const uint32_t q = bit_exp_dev<VARIANT, false>(x[s][e], lower, mx, P);
                    x[s][e] = (int32_t)q;
                    sum += q;
                }
        } else {
#pragma unroll
            for (int s = 0; s < SLOTS; ++s)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const uint32_t q = bit_exp_dev<VARIANT, true>(x[s][e], lower, mx, P);
                    x[s][e] = (int32_t)q;
                    sum += q;
                }
        }
        sum = row_sum(sum);
        const uint32_t f = floor_pow2_div(P.m_bits, sum);
        const uint32_t f_top = P.p_shift <= 24 ? f << (24 - P.p_shift) : 0u;
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            if (POSTMODE == PM_GENERAL && P.p_shift <= 24)
                w[s] = post_lut_gather(lut, normalise4<PM_NONE>((uint32_t)x[s][0], (uint32_t)x[s][1],
                                                                (uint32_t)x[s][2], (uint32_t)x[s][3], f, f_top, P));
            else
                w[s] = normalise4<POSTMODE>((uint32_t)x[s][0], (uint32_t)x[s][1], (uint32_t)x[s][2],
                                            (uint32_t)x[s][3], f, f_top, P);
        }
    }
}

// Instrumented build (`python -m paper_2511_15369_amd.build timeline` -> libiptq_timeline.so; read
// with `python -m paper_2511_15369_amd.timeline`): each wavefront records the device-wide clock
// at entry, when its slab has landed in LDS, after the arithmetic, after its last store is
// issued and after that store is acknowledged, for the first kTimelineSlabs slabs of a launch.
#ifdef IPTQ_TIMELINE
constexpr int kTimelineSlabs = 65536;
static __device__ uint64_t g_timeline[5 * kTimelineSlabs];
#define IPTQ_TL(k, t) do { if (lane == 0 && slab < kTimelineSlabs) g_timeline[5 * slab + (k)] = (t); } while (0)
#else
#define IPTQ_TL(k, t) do { } while (0)
#endif

// MASKKIND: 0 no per-window mask, 1 the int32 table read beside the bias, 2 one bit per key.
template <int COLS, int K, int MODE, bool BIAS, int POSTMODE, int MASKKIND, bool PRE = false>
IPTQ_DEV void softmax_rows_body(const SoftmaxBatch &B)
{
    constexpr bool MASK = MASKKIND == 1;
#ifdef IPTQ_TIMELINE
    const uint64_t t_entry = wall_clock64();
#endif
    constexpr int RPW = 64 / K;                       // rows per wavefront
    constexpr int SLAB = RPW * COLS;                  // elements per slab
    static_assert(RPW % 4 == 0, "slab must start on a 16-byte boundary of the int32 input");
    // 16-byte blocks a row can touch: rows start at element offsets that are multiples of
    // gcd(COLS, 4) inside a block
    constexpr int NB = (COLS % 4 == 0) ? COLS / 4 : ((COLS % 2 == 0) ? (COLS + 2 + 3) / 4 : (COLS + 3 + 3) / 4);
    constexpr int SLOTS = (NB + K - 1) / K;           // blocks per lane
    constexpr int IN_CHUNKS = SLAB / 4;               // 16-byte chunks of the input slab
    constexpr bool OUT16 = SLAB % 16 == 0;            // output slab is whole 16-byte chunks
    constexpr int OUT_CHUNKS = OUT16 ? SLAB / 16 : SLAB / 4;   // else whole dwords
    __shared__ __attribute__((aligned(16))) uint8_t lds_all[kRowsWpb][SLAB * 4];
    __shared__ uint8_t lut_all[kRowsWpb][POSTMODE == PM_GENERAL ? kPostLutBytes : 4];

    touch_kernel_arguments<8 + sizeof(SoftmaxItem)>();   // the batch header and its first problem
    const int lane = threadIdx.x & 63;
    // (the wavefront index as a scalar: everything derived from it - the slab, its table offsets,
    // the runs of mask entries - is then computed on the scalar unit)
    const int wv = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    int it = 0;                                       // which problem this workgroup serves
    for (int i = 1; i < B.n_items; ++i)
        if (blockIdx.x >= B.item[i].first_wg) it = i;
    const SoftmaxItem &I = B.item[it];
    const SoftmaxDev P = I.P;                         // by value: every field loaded once, up front
    const int32_t *__restrict__ scores = I.scores;
    const int32_t *__restrict__ bias = I.bias;
    uint8_t *__restrict__ out = I.out;
    static_assert(!MASK || RPW <= COLS, "a slab may cross one wrap of the query index at most");
    constexpr int MW = MASKKIND == 2 ? (COLS + 63) / 64 : 1;   // 64-bit words of packed mask per query
    const uint32_t lw = blockIdx.x - I.first_wg;
    int64_t slab = (int64_t)lw * kRowsWpb + wv;
    if (BIAS && I.share_q != 0) {
        const uint32_t g = mulhi_u32(lw, I.share_magic) >> I.share_sh;
        slab = (int64_t)g * (kRowsWpb * I.share_q) + (uint32_t)wv * I.share_q + (lw - g * I.share_q);
    }
    if (slab >= I.n_slabs) return;                    // no workgroup barrier below

#ifdef IPTQ_TIMELINE
    IPTQ_TL(0, t_entry);
#endif
    uint8_t *lds = lds_all[wv];
    uint8_t *lut = lut_all[wv];
    if (POSTMODE == PM_GENERAL) {                     // ordered before its use by the fences below
        const int p_max = 1 << (P.m_bits - P.p_shift);    // 2^(b-1) <= 128
        for (int p = lane; p <= p_max; p += 64) lut[p] = (uint8_t)post_dev<PM_GENERAL>((uint32_t)p, P);
    }
    const int32_t *src = scores + slab * SLAB;       // anywhere on the 4-byte grid
    const int lr = lane / K;                          // row inside the slab
    const int j = lane % K;                           // lane inside the row
    const int e_r = lr * COLS;                        // first element of the row in the slab
    const int b_r = e_r >> 2;                         // its 16-byte block
    const int phi = e_r & 3;                          // and its offset inside that block

    // ---- the packed mask: this lane's row takes the words of [window, query]; loaded now, used
    // after the slab has been read back from LDS
    uint64_t mask_words[MW] = {};
    if (MASKKIND == 2) {
        const uint32_t row = (uint32_t)(slab * RPW) + (uint32_t)lr;
        uint32_t rm = 0;
        if (P.mask_period_rows >= 2)
            rm = row - (mulhi_u32(row, P.mperiod_magic) >> P.mperiod_sh) * (uint32_t)P.mask_period_rows;
        const uint32_t w = P.group_rows >= 2 ? mulhi_u32(rm, P.group_magic) >> P.group_sh : rm;
        const uint32_t q = (rm - w * (uint32_t)P.group_rows) % (uint32_t)COLS;
        const uint64_t *mw = I.mask_bits + (uint64_t)(w * (uint32_t)COLS + q) * MW;
#pragma unroll
        for (int i = 0; i < MW; ++i) mask_words[i] = mw[i];
    }

    // ---- flat copy of the slab into LDS, bias added on the way.  A partial last slab (the
    // tensor's row count is not a multiple of RPW) reads nothing beyond its last valid
    // element and zero-fills the rest; its surplus rows are computed and never stored.
    const bool partial = I.tail_rows != 0 && slab == I.n_slabs - 1;
    const int valid_el = (partial ? I.tail_rows : RPW) * COLS;
    // STRADDLE: the additive table's size is not a multiple of four scores and its end falls
    // inside this slab, so one of the slab's chunks takes entries from both ends of the table.
    uint32_t boff = 0;
    if (BIAS) boff = row_mod_period((uint32_t)(slab * RPW), P) * (uint32_t)COLS;
    const uint32_t pe = (uint32_t)P.bias_period_rows * (uint32_t)COLS;
    const bool straddle = BIAS && (pe & 3u) != 0 && boff + (uint32_t)SLAB > pe;    // wavefront-uniform
    // the per-window mask: at most two runs of entries (MaskRuns)
    MaskRuns MR = {};
    if (MASK) MR = mask_runs_of_slab<COLS, RPW>(I.mask, (uint32_t)(slab * RPW), P);
    // EXACT: the bias is added with the minus-infinity rule per score (four lane-ops).  Otherwise
    // with the saturating sum alone, which is the same value unless a score or a table entry is
    // INT32_MIN; the smallest operand is tracked beside it (two lane-ops per score in all), and
    // the function returns whether any lane of the wavefront met INT32_MIN, in which case the
    // caller runs the exact form over the slab again.
    auto copy_in = [&](auto tag, auto straddle_tag, auto exact_tag) -> bool {
        constexpr bool PARTIAL = decltype(tag)::value;
        constexpr bool STRADDLE = decltype(straddle_tag)::value;
        constexpr bool EXACT = decltype(exact_tag)::value;
        i32x4 lowest = {0, 0, 0, 0};
        i32x4 *lds4 = reinterpret_cast<i32x4 *>(lds);
        i32x4 first4 = {0, 0, 0, 0};
        if (BIAS && STRADDLE) first4 = load_i32x4(bias);
        constexpr int NPASS = (IN_CHUNKS + 63) / 64;
        // With the mask there are three loads per chunk, more than the registers hold in flight
        // at once: the scores (the loads that go to HBM) are all issued first, the two tables'
        // entries (cache hits) follow pass by pass.
        i32x4 sv[MASK ? NPASS : 1];
        if (MASK) {
#pragma unroll
            for (int i = 0; i < NPASS; ++i) {
                const int idx = i * 64 + lane;
                const bool full_pass = (i + 1) * 64 <= IN_CHUNKS;
                const int li = (PARTIAL || full_pass) ? idx : min(idx, IN_CHUNKS - 1);
                if (!PARTIAL || 4 * idx + 3 < valid_el) {
                    sv[i] = stream_load_i32x4(src + 4 * li);
                } else {
                    const int32_t *s = src + 4 * idx;
                    sv[i] = (i32x4){0, 0, 0, 0};
                    if (4 * idx < valid_el) sv[i].x = s[0];
                    if (4 * idx + 1 < valid_el) sv[i].y = s[1];
                    if (4 * idx + 2 < valid_el) sv[i].z = s[2];
                }
            }
        }
#pragma unroll
        for (int i = 0; i < NPASS; ++i) {
            const int idx = i * 64 + lane;
            const bool full_pass = (i + 1) * 64 <= IN_CHUNKS;
            if (PARTIAL && !(full_pass || idx < IN_CHUNKS)) continue;
            // In the last, partly filled pass the lanes beyond the slab load its last chunk again
            // and write it to the same LDS address again (same data): a load behind a
            // lane-divergent branch would be issued after all the others had returned, a second
            // memory round trip per wavefront.
            const int li = (PARTIAL || full_pass) ? idx : min(idx, IN_CHUNKS - 1);
            i32x4 v;
            if (MASK) {
                v = sv[i];
            } else if (!PARTIAL || 4 * idx + 3 < valid_el) {
                v = stream_load_i32x4(src + 4 * li);
            } else {
                const int32_t *s = src + 4 * idx;
                v = (i32x4){0, 0, 0, 0};
                if (4 * idx < valid_el) v.x = s[0];
                if (4 * idx + 1 < valid_el) v.y = s[1];
                if (4 * idx + 2 < valid_el) v.z = s[2];
            }
            i32x4 bv = {0, 0, 0, 0};
            if (BIAS) {
                uint32_t o = boff + 4u * (uint32_t)li;
                if (o >= pe) o -= pe;
                bv = STRADDLE ? bias_chunk_wrapping(bias, o, pe, first4) : load_i32x4_at(bias, 4u * o);   // table below 4 GiB
            }
            if (MASK) {
                const i32x4 mv = mask_chunk(I.mask, MR, 4u * (uint32_t)li);
                if (BIAS) {
                    v.x = add_two_table_entries(v.x, bv.x, mv.x);
                    v.y = add_two_table_entries(v.y, bv.y, mv.y);
                    v.z = add_two_table_entries(v.z, bv.z, mv.z);
                    v.w = add_two_table_entries(v.w, bv.w, mv.w);
                } else {
                    v = add_table_chunk(v, mv);
                }
            } else if (BIAS) {
                if (EXACT) {
                    v = add_table_chunk(v, bv);
                } else {
                    lowest.x = min(min(lowest.x, v.x), bv.x);
                    lowest.y = min(min(lowest.y, v.y), bv.y);
                    lowest.z = min(min(lowest.z, v.z), bv.z);
                    lowest.w = min(min(lowest.w, v.w), bv.w);
                    v.x = sat_add_i32(v.x, bv.x);
                    v.y = sat_add_i32(v.y, bv.y);
                    v.z = sat_add_i32(v.z, bv.z);
                    v.w = sat_add_i32(v.w, bv.w);
                }
            }
            lds4[li] = v;
        }
        wave_lds_fence();
        return !EXACT &&
               __builtin_amdgcn_ballot_w64(min(min(lowest.x, lowest.y), min(lowest.z, lowest.w)) == kI32Min) != 0;
    };
    // a partial slab and a per-window table take the exact form at once
    constexpr bool FAST_ADD = BIAS && !MASK;
    bool redo = false;                                // wavefront-uniform
    // (the rare forms are marked so that the compiler lays the common path out contiguously: every
    // launch starts with a cold instruction cache)
    if (__builtin_expect(partial, 0)) copy_in(std::true_type{}, std::integral_constant<bool, BIAS>{}, std::true_type{});
    else if (__builtin_expect(straddle, 0)) redo = copy_in(std::false_type{}, std::true_type{}, std::integral_constant<bool, !FAST_ADD>{});
    else redo = copy_in(std::false_type{}, std::false_type{}, std::integral_constant<bool, !FAST_ADD>{});
    if (FAST_ADD && __builtin_expect(redo, 0)) {
        // Some score or table entry of this slab is INT32_MIN: the slab once more with the exact
        // addition, one chunk at a time (a rare path: it must cost no registers, not no time).
        i32x4 *lds4 = reinterpret_cast<i32x4 *>(lds);
        const i32x4 first4 = load_i32x4(bias);
#pragma unroll 1
        for (int i = 0; i < (IN_CHUNKS + 63) / 64; ++i) {
            const int li = min(i * 64 + lane, IN_CHUNKS - 1);
            const i32x4 v = stream_load_i32x4(src + 4 * li);
            uint32_t o = boff + 4u * (uint32_t)li;
            if (o >= pe) o -= pe;
            const i32x4 bv = straddle ? bias_chunk_wrapping(bias, o, pe, first4) : load_i32x4(bias + o);
            lds4[li] = add_table_chunk(v, bv);
        }
        wave_lds_fence();
    }

    IPTQ_TL(1, wall_clock64());
    // ---- this lane's blocks; elements outside the row become "minus infinity"
    int32_t x[SLOTS][4];
#pragma unroll
    for (int s = 0; s < SLOTS; ++s) {
        const int b = s * K + j;
        const bool always_inside = 4 * (s * K + K - 1) < COLS;
        // a block beyond the row's last one is read from the last one and masked entirely below
        // (no lane-divergent branch around the LDS read)
        const int bb = always_inside ? b : min(b, ((phi + COLS + 3) >> 2) - 1);
        const i32x4 v = reinterpret_cast<const i32x4 *>(lds)[b_r + bb];
        x[s][0] = v.x; x[s][1] = v.y; x[s][2] = v.z; x[s][3] = v.w;
        const bool may_cut = (s == 0) || (4 * (s * K + K - 1) + 3 >= COLS);
        if (may_cut) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int c = 4 * b + e - phi;
                if ((unsigned)c >= (unsigned)COLS) x[s][e] = kI32Min;
            }
        }
    }
    wave_lds_fence();                                 // the slab area is reused for the output

    if (MASKKIND == 2) {
        // element e of slot s is key 4 (s K + j) + e - phi: shift the row's bits once, by
        // sh = 4 j - phi in [-3, 4 K - 1], so that this bit sits at the compile-time position
        // 4 s K + e (keys below 0 and beyond the row read zeros; those elements are minus infinity
        // already).  Word i of the shifted string is bits [sh', sh' + 63] of two neighbouring words.
        const int sh = 4 * j - phi;
        const bool back = sh < 0;
        const int sh6 = sh & 63;
        uint64_t aligned[MW];
#pragma unroll
        for (int i = 0; i < MW; ++i) {
            const uint64_t prev = i > 0 ? mask_words[i - 1] : 0, cur = mask_words[i];
            const uint64_t next = i + 1 < MW ? mask_words[i + 1] : 0;
            const uint64_t lo64 = back ? prev : cur, hi64 = back ? cur : next;
            aligned[i] = sh6 == 0 ? lo64 : (lo64 >> sh6) | (hi64 << (64 - sh6));
        }
#pragma unroll
        for (int s = 0; s < SLOTS; ++s)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int pos = 4 * s * K + e;
                if (pos >= 64 * MW) continue;         // beyond the words: keys past the row
                const uint64_t wd = aligned[pos >> 6];
                const uint32_t half = (pos & 32) ? (uint32_t)(wd >> 32) : (uint32_t)wd;
                const uint32_t m = (uint32_t)__builtin_amdgcn_sbfe((int32_t)half, pos & 31, 1);   // all ones: masked
                x[s][e] = select_bits_i32(m, kI32Min, x[s][e]);
            }
    }

    uint32_t w[SLOTS];                                // four output bytes per block
    bool done = false;                                // wavefront-uniform
    // ---- fused requantization of the scores, folded into Eq. 6 (PRE instantiations, parameters
    // with SoftmaxDev::pre_rowconst): the maximum is taken over the raw scores (the
    // requantization is monotone), each delta costs one 24-bit multiply-add and a shift.  Rows
    // whose raw maximum lies within pre_dmax of INT32_MIN (the clamp could not tell their masked
    // entries from live ones) send the wavefront down the ordinary route below.
    if (PRE && P.pre_rowconst != 0) {
        int32_t mr = kI32Min;
#pragma unroll
        for (int s = 0; s < SLOTS; ++s)
#pragma unroll
            for (int e = 0; e < 4; ++e) mr = max(mr, x[s][e]);
        mr = group_max_i32<K>(mr);
        const bool low = ((uint32_t)mr ^ 0x80000000u) < P.pre_dmax;        // mr - INT32_MIN as unsigned
        if (__builtin_expect(__builtin_amdgcn_ballot_w64(low) == 0, 1)) {
            const int64_t t = (int64_t)mr * (int64_t)P.pre_m + ((int64_t)1 << (P.pre_s - 1));
            const uint32_t smask = (1u << P.pre_s) - 1u;                   // pre_s <= 31 here
            const uint32_t c_row = smask - ((uint32_t)t & smask);
            if (P.variant == 0)
                softmax_slab_math<K, SLOTS, MODE, 0, POSTMODE, LaneGroupSum<K>, true>(x, w, mr, 0, false, lut, P, LaneGroupSum<K>(), c_row);
            else
                softmax_slab_math<K, SLOTS, MODE, 1, POSTMODE, LaneGroupSum<K>, true>(x, w, mr, 0, false, lut, P, LaneGroupSum<K>(), c_row);
            done = true;
        }
    }
    if (!done) {
    // ---- fused requantization of the scores (after the bias, before the maximum).  Done on
    // the registers, not in the copy loop, so that every load of the slab stays in flight;
    // computed for every element and selected, so that it compiles without branches.
    if (P.pre_mode == 1) {
        const int32_t pre_mul = P.pre_mul, pre_sh2 = P.pre_sh2;
        const int64_t pre_rnd = P.pre_rnd;
#pragma unroll
        for (int s = 0; s < SLOTS; ++s)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int32_t r = pre_requant_narrow(x[s][e], pre_mul, pre_rnd, pre_sh2);
                x[s][e] = x[s][e] == kI32Min ? kI32Min : r;
            }
    } else if (P.pre_mode == 2) {                     // shifts below 16: the general 64-bit form
        const int32_t pre_m = P.pre_m, pre_s = P.pre_s;
#pragma unroll
        for (int s = 0; s < SLOTS; ++s)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int32_t r = pre_requant_dev(x[s][e], pre_m, pre_s);
                x[s][e] = x[s][e] == kI32Min ? kI32Min : r;
            }
    }

    // ---- Eq. 6: row maximum
    int32_t mx = kI32Min;
#pragma unroll
    for (int s = 0; s < SLOTS; ++s)
#pragma unroll
        for (int e = 0; e < 4; ++e) mx = max(mx, x[s][e]);
    mx = group_max_i32<K>(mx);

    // Rows whose maximum lies within D of INT32_MIN cannot rely on the clamp to zero out
    // masked entries; the whole wavefront then takes the 32-bit path with an explicit test.
    const int32_t D = P.d_clamp;
    const bool low_row = mx < kI32Min + D;
    const int32_t lower = low_row ? kI32Min : mx - D;
    const bool any_low = __builtin_amdgcn_ballot_w64(low_row) != 0;

    if (P.variant == 0) softmax_slab_math<K, SLOTS, MODE, 0, POSTMODE>(x, w, mx, lower, any_low, lut, P);
    else if (P.variant == 1) softmax_slab_math<K, SLOTS, MODE, 1, POSTMODE>(x, w, mx, lower, any_low, lut, P);
    else softmax_slab_math<K, SLOTS, MODE, 2, POSTMODE>(x, w, mx, lower, any_low, lut, P);
    }
    if (POSTMODE == PM_NONE && P.post_xor != 0) {     // signed output around the zero-point -128
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) w[s] ^= P.post_xor;
    }

    IPTQ_TL(2, wall_clock64());
    // ---- assemble the slab's bytes in LDS
    uint32_t *lds32 = reinterpret_cast<uint32_t *>(lds);
#pragma unroll
    for (int s = 0; s < SLOTS; ++s) {
        const int b = s * K + j;
        const bool always_full = (s != 0) && (4 * (s * K + K - 1) + 3 < COLS);
        if (always_full) {
            lds32[b_r + b] = w[s];
        } else {
            const int c0 = 4 * b - phi;
            if (c0 >= 0 && c0 + 3 < COLS) {
                lds32[b_r + b] = w[s];
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if ((unsigned)(c0 + e) < (unsigned)COLS)
                        lds[4 * (b_r + b) + e] = (uint8_t)(w[s] >> (8 * e));
            }
        }
    }
    wave_lds_fence();

    // ---- flat, fully coalesced store (byte stores at the end of a partial slab)
    auto copy_out = [&](auto tag) {
        constexpr bool PARTIAL = decltype(tag)::value;
        constexpr int CB = OUT16 ? 16 : 4;            // bytes per store
        uint8_t *dst8 = out + slab * SLAB;
#pragma unroll
        for (int i = 0; i < (OUT_CHUNKS + 63) / 64; ++i) {
            const int idx = i * 64 + lane;
            if ((i + 1) * 64 <= OUT_CHUNKS || idx < OUT_CHUNKS) {
                if (!PARTIAL || CB * idx + CB - 1 < valid_el) {
                    if (OUT16)
                        stream_store_bytes16(reinterpret_cast<const u32x4 *>(lds)[idx], dst8 + 16 * idx);
                    else
                        stream_store_bytes4(lds32[idx], dst8 + 4 * idx);
                } else {
#pragma unroll 1
                    for (int b = CB * idx; b < valid_el && b < CB * idx + CB; ++b) dst8[b] = lds[b];
                }
            }
        }
    };
    if (__builtin_expect(partial, 0)) copy_out(std::true_type{});
    else copy_out(std::false_type{});
#ifdef IPTQ_TIMELINE
    IPTQ_TL(3, wall_clock64());
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    IPTQ_TL(4, wall_clock64());
#endif
}

template <int COLS, int K, int MODE, bool BIAS, int POSTMODE>
__global__ void __launch_bounds__(64 * kRowsWpb)
softmax_rows_kernel(SoftmaxBatch B)
{
    softmax_rows_body<COLS, K, MODE, BIAS, POSTMODE, 0>(B);
}

// The same with the per-window mask beside the bias: three loads per chunk.  Compiled for five
// wavefronts per SIMD instead of the six the LDS staging would allow, so that a wavefront has
// the registers to keep all its loads in flight at once.
template <int COLS, int K, int MODE, int POSTMODE>
__global__ void __launch_bounds__(64 * kRowsWpb) __attribute__((amdgpu_waves_per_eu(4, 5)))
softmax_rows_masked_kernel(SoftmaxBatch B)
{
    softmax_rows_body<COLS, K, MODE, true, POSTMODE, 1>(B);
}

// The mask one bit per key: one to three 8-byte loads per lane (49- and 144-token windows) and
// two instructions per score instead of a third table.
template <int COLS, int K, int MODE, int POSTMODE>
__global__ void __launch_bounds__(64 * kRowsWpb)
softmax_rows_maskbits_kernel(SoftmaxBatch B)
{
    softmax_rows_body<COLS, K, MODE, true, POSTMODE, 2>(B);
}

// The same with the requantization of the scores folded into Eq. 6 where the parameters allow it
// (no tables, packed arithmetic, identity or clip post step).
template <int COLS, int K, int MODE, int POSTMODE>
__global__ void __launch_bounds__(64 * kRowsWpb)
softmax_rows_requant_kernel(SoftmaxBatch B)
{
    softmax_rows_body<COLS, K, MODE, false, POSTMODE, 0, true>(B);
}

// Launch helper, defined once per row length in softmax_rows_<cols>.hip so that the
// instantiations compile in parallel.  mode: 0 / 1 / 2 as above; all items share has_bias and
// has_mask; fold_pre: some item has SoftmaxDev::pre_rowconst.
template <int COLS, int K>
hipError_t launch_softmax_rows(const SoftmaxBatch &B, unsigned total_wgs, bool has_bias, int mask_kind,
                               bool fold_pre, int mode, int post_mode, hipStream_t stream);

// The compiled row lengths with their lanes per row: ViT / DeiT at 224^2 (197; 198 with a
// distillation token), Swin 7x7 and 12x12 windows (49, 144), ViT-L/14 (257), 384^2 / 16 (577).
// Each is instantiated in its own softmax_rows_<cols>.hip.
#define IPTQ_ROWS_SHAPES(X) X(197, 4) X(49, 2) X(198, 4) X(144, 4) X(257, 8) X(577, 16)
// More lanes per row shorten a wavefront's arithmetic chain (less exposed time at the start
// and the end of a launch) and cost some idle lanes in steady state: measured on MI355X they
// win for launches up to about 1.5 ViT-B layers and lose beyond, so launches of at most
// kRowsAltMaxElements elements use these instead (softmax_rows_<cols>_k<K>.hip).
#define IPTQ_ROWS_SHAPES_ALT(X) X(197, 8) X(198, 8)
constexpr int64_t kRowsAltMaxElements = 90 * 1000 * 1000;
// The per-window mask is compiled in for the window sizes of shifted-window attention only
// (7 x 7 and 12 x 12 tokens), with the bias table beside it.
constexpr bool rows_mask_compiled(int cols) { return cols == 49 || cols == 144; }
constexpr bool rows_maskbits_compiled(int cols) { return cols == 49 || cols == 144; }
#define IPTQ_DECLARE_ROWS_LAUNCHER(COLS, K)                                                       \
    template <>                                                                                   \
    hipError_t launch_softmax_rows<COLS, K>(const SoftmaxBatch &, unsigned, bool, int, bool, int, int, hipStream_t);
IPTQ_ROWS_SHAPES(IPTQ_DECLARE_ROWS_LAUNCHER)
IPTQ_ROWS_SHAPES_ALT(IPTQ_DECLARE_ROWS_LAUNCHER)

#define IPTQ_ROWS_LAUNCH(COLS, K, MODE, BIAS, PM, MASK)                                           \
    do {                                                                                          \
        if constexpr (MASK == 1)                                                                  \
            hipLaunchKernelGGL((softmax_rows_masked_kernel<COLS, K, MODE, PM>), grid, block, 0, stream, B);   \
        else if constexpr (MASK == 2)                                                             \
            hipLaunchKernelGGL((softmax_rows_maskbits_kernel<COLS, K, MODE, PM>), grid, block, 0, stream, B); \
        else                                                                                      \
            hipLaunchKernelGGL((softmax_rows_kernel<COLS, K, MODE, BIAS, PM>), grid, block, 0, stream, B);    \
    } while (0)

template <int COLS, int K, bool BIAS, int MASK>
static hipError_t launch_rows_b(const SoftmaxBatch &B, unsigned total_wgs, int mode, int post_mode,
                                hipStream_t stream)
{
    const dim3 grid(total_wgs), block(64 * kRowsWpb);
#define IPTQ_ROWS_LAUNCH_PM(MODE)                                                                 \
    switch (post_mode) {                                                                          \
    case PM_NONE: IPTQ_ROWS_LAUNCH(COLS, K, MODE, BIAS, PM_NONE, MASK); break;                    \
    case PM_CLAMP127: IPTQ_ROWS_LAUNCH(COLS, K, MODE, BIAS, PM_CLAMP127, MASK); break;            \
    default: IPTQ_ROWS_LAUNCH(COLS, K, MODE, BIAS, PM_GENERAL, MASK); break;                      \
    }
    if (mode == 0) { IPTQ_ROWS_LAUNCH_PM(0) }
    else if (mode == 1) { IPTQ_ROWS_LAUNCH_PM(1) }
    else { IPTQ_ROWS_LAUNCH_PM(2) }
#undef IPTQ_ROWS_LAUNCH_PM
    return hipGetLastError();
}

template <int COLS, int K>
static hipError_t launch_rows_requant(const SoftmaxBatch &B, unsigned total_wgs, int mode, int post_mode,
                                      hipStream_t stream)
{
    const dim3 grid(total_wgs), block(64 * kRowsWpb);
    if (mode == 1 && post_mode == PM_NONE)
        hipLaunchKernelGGL((softmax_rows_requant_kernel<COLS, K, 1, PM_NONE>), grid, block, 0, stream, B);
    else if (mode == 1)
        hipLaunchKernelGGL((softmax_rows_requant_kernel<COLS, K, 1, PM_CLAMP127>), grid, block, 0, stream, B);
    else if (post_mode == PM_NONE)
        hipLaunchKernelGGL((softmax_rows_requant_kernel<COLS, K, 2, PM_NONE>), grid, block, 0, stream, B);
    else
        hipLaunchKernelGGL((softmax_rows_requant_kernel<COLS, K, 2, PM_CLAMP127>), grid, block, 0, stream, B);
    return hipGetLastError();
}

template <int COLS, int K>
static hipError_t launch_rows_masked(const SoftmaxBatch &B, unsigned total_wgs, int mask_kind, int mode,
                                     int post_mode, hipStream_t stream)
{
    if constexpr (rows_mask_compiled(COLS)) {
        if (mask_kind == 1) return launch_rows_b<COLS, K, true, 1>(B, total_wgs, mode, post_mode, stream);
    }
    if constexpr (rows_maskbits_compiled(COLS)) {
        if (mask_kind == 2) return launch_rows_b<COLS, K, true, 2>(B, total_wgs, mode, post_mode, stream);
    }
    return hipErrorInvalidValue;                      // the dispatcher never asks for it
}

#ifdef IPTQ_TIMELINE
// copies the timestamps of the last launches of this translation unit's kernels to the host
#define IPTQ_DEFINE_TIMELINE_READER(COLS, K)                                                      \
    extern "C" int iptq_debug_timeline_##COLS##_##K(uint64_t *host, int n)                        \
    {                                                                                             \
        if (!host || n < 0 || n > 5 * kTimelineSlabs) return IPTQ_ERR_SHAPE;                      \
        return hipMemcpyFromSymbol(host, HIP_SYMBOL(g_timeline), (size_t)n * 8) == hipSuccess ? IPTQ_OK : IPTQ_ERR_HIP;  \
    }
#else
#define IPTQ_DEFINE_TIMELINE_READER(COLS, K)
#endif

#define IPTQ_DEFINE_ROWS_LAUNCHER(COLS, K)                                                        \
    IPTQ_DEFINE_TIMELINE_READER(COLS, K)                                                          \
    template <>                                                                                   \
    hipError_t launch_softmax_rows<COLS, K>(const SoftmaxBatch &B, unsigned total_wgs,            \
                                            bool has_bias, int mask_kind, bool fold_pre,          \
                                            int mode, int post_mode, hipStream_t stream)          \
    {                                                                                             \
        if (mask_kind != 0)                                                                       \
            return launch_rows_masked<COLS, K>(B, total_wgs, mask_kind, mode, post_mode, stream); \
        if (fold_pre && !has_bias && mode != 0 && post_mode != PM_GENERAL)                        \
            return launch_rows_requant<COLS, K>(B, total_wgs, mode, post_mode, stream);           \
        return has_bias ? launch_rows_b<COLS, K, true, 0>(B, total_wgs, mode, post_mode, stream)         \
                        : launch_rows_b<COLS, K, false, 0>(B, total_wgs, mode, post_mode, stream);       \
    }

}  // namespace iptq
