// Integer softmax for gfx950 (Section 4.4, Eq. 6-15): the any-row-length kernel and the
// dispatch between it and the fixed-row-length kernels of softmax_rows.h.
//   softmax_generic_kernel - run-time row length, one wavefront per row, three passes.
//                          Serves odd shapes, the tail rows of the fixed-length kernels and
//                          the fused pre-requantization.
#include <hip/hip_runtime.h>

#include "../../include/iptq.h"
#include "device_common.h"
#include "kernels.h"
#include "plan.h"
#include "softmax_rows.h"

namespace iptq {

// ---------------------------------------------------------------------------------------
// Any row length: one wavefront per row, three passes over the row (maximum, sum of
// exponentials, normalise).  The row is re-read from global memory in each pass; a row of
// a few hundred scores stays in the L1/L2 cache between passes.
template <int VARIANT>
__global__ void __launch_bounds__(256)
softmax_generic_kernel(const int32_t *__restrict__ scores, const int32_t *__restrict__ bias,
                       const int32_t *__restrict__ mask, const uint64_t *__restrict__ mask_bits,
                       uint8_t *__restrict__ out, int64_t row_begin, int64_t row_end, int32_t cols,
                       int32_t has_bias, int32_t has_pre, SoftmaxDev P)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = row_begin + (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= row_end) return;
    const int32_t *srow = scores + row * cols;
    const int32_t *brow = nullptr;
    if (has_bias) brow = bias + (int64_t)row_mod_period((uint32_t)row, P) * cols;
    const int32_t *mrow = nullptr;
    const uint64_t *mbits = nullptr;                  // the row's mask one bit per key
    if (mask || mask_bits) {
        // rows are ordered [image, window, head, query]: window (r mod period) div (heads * cols),
        // query (r mod (heads * cols)) mod cols; cols is a run-time value here, so the last one is
        // a subtraction loop over the heads in front (once per row)
        const uint32_t r = (uint32_t)row;
        uint32_t rm = 0;
        if (P.mask_period_rows >= 2)
            rm = r - (mulhi_u32(r, P.mperiod_magic) >> P.mperiod_sh) * (uint32_t)P.mask_period_rows;
        const uint32_t w = P.group_rows >= 2 ? mulhi_u32(rm, P.group_magic) >> P.group_sh : rm;
        uint32_t q = rm - w * (uint32_t)P.group_rows;
        while (q >= (uint32_t)cols) q -= (uint32_t)cols;
        if (mask) mrow = mask + ((int64_t)w * cols + q) * cols;
        else mbits = mask_bits + ((int64_t)w * cols + q) * ((cols + 63) >> 6);
    }

    auto fetch = [&](int c) -> int32_t {
        int32_t v = srow[c];
        if (has_bias) v = add_table_entry(v, brow[c]);
        if (mrow) v = add_table_entry(v, mrow[c]);
        if (mbits && ((mbits[c >> 6] >> (c & 63)) & 1)) v = kI32Min;
        if (has_pre && v != kI32Min) v = pre_requant_dev(v, P.pre_m, P.pre_s);
        return v;
    };

    int32_t mx = kI32Min;
    for (int c = lane; c < cols; c += 64) mx = max(mx, fetch(c));
    mx = wave_max_i32(mx);

    const int32_t D = P.d_clamp;
    const int32_t lower = (mx < kI32Min + D) ? kI32Min : mx - D;
    uint32_t sum = 0;
    for (int c = lane; c < cols; c += 64) sum += bit_exp_dev<VARIANT, true>(fetch(c), lower, mx, P);
    sum = wave_sum_u32(sum);

    const uint32_t f = floor_pow2_div(P.m_bits, sum);
    uint8_t *orow = out + row * cols;
    for (int c = lane; c < cols; c += 64) {
        const uint32_t q = bit_exp_dev<VARIANT, true>(fetch(c), lower, mx, P);
        const uint32_t p = (q * f) >> P.p_shift;
        orow[c] = (uint8_t)post_dev<PM_GENERAL>(p, P);
    }
}

// ---------------------------------------------------------------------------------------
// A 0 / INT32_MIN window mask as one bit per key: thread x = query row, block y = word of that
// row; each thread reads up to 64 entries of its mask row.  Run once per model (a few hundred
// kilobytes), not on the inference path.
__global__ void __launch_bounds__(256)
pack_window_mask_kernel(const int32_t *__restrict__ mask, int64_t n_queries, int32_t cols,
                        int32_t words, uint64_t *__restrict__ bits)
{
    const int64_t row = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (row >= n_queries) return;
    const int32_t wd = (int32_t)blockIdx.y;
    const int32_t *m = mask + row * cols;
    const int32_t k0 = wd * 64;
    const int32_t k1 = min(cols, k0 + 64);
    uint64_t w = 0;
    for (int32_t k = k0; k < k1; ++k)
        if (m[k] == kI32Min) w |= (uint64_t)1 << (k - k0);
    bits[row * words + wd] = w;
}

hipError_t pack_window_mask_dispatch(const int32_t *mask, int64_t n_queries, int32_t cols, uint64_t *bits,
                                     hipStream_t stream)
{
    const int32_t words = (cols + 63) / 64;           // at most 1024
    if (n_queries <= 0) return hipSuccess;
    hipLaunchKernelGGL(pack_window_mask_kernel, dim3((unsigned)((n_queries + 255) / 256), (unsigned)words),
                       dim3(256), 0, stream, mask, n_queries, cols, words, bits);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Host-side dispatch.

static int post_mode_of(const SoftmaxDev &P, int out_bits)
{
    if (P.post_xor != 0) return PM_NONE;              // p - 128: one exclusive-or on the packed bytes
    const bool identity = P.post_m == 1 && P.post_s == 0 && P.post_zp == 0 && P.qmin <= 0;
    if (!identity) return PM_GENERAL;
    if (P.qmax >= (1 << (out_bits - 1))) return PM_NONE;
    return (P.qmax == 127 && out_bits == 8) ? PM_CLAMP127 : PM_GENERAL;
}

static hipError_t launch_generic(const int32_t *scores, const int32_t *bias, const int32_t *mask,
                                 const uint64_t *mask_bits, uint8_t *out, int64_t row_begin, int64_t row_end, int32_t cols,
                                 bool has_bias, bool has_pre, const SoftmaxDev &P, hipStream_t stream)
{
    const int64_t n = row_end - row_begin;
    if (n <= 0) return hipSuccess;
    const dim3 grid((unsigned)((n + 3) / 4)), block(256);
    if (P.variant == 0)
        hipLaunchKernelGGL(softmax_generic_kernel<0>, grid, block, 0, stream, scores, bias, mask, mask_bits, out,
                           row_begin, row_end, cols, (int32_t)has_bias, (int32_t)has_pre, P);
    else if (P.variant == 1)
        hipLaunchKernelGGL(softmax_generic_kernel<1>, grid, block, 0, stream, scores, bias, mask, mask_bits, out,
                           row_begin, row_end, cols, (int32_t)has_bias, (int32_t)has_pre, P);
    else
        hipLaunchKernelGGL(softmax_generic_kernel<2>, grid, block, 0, stream, scores, bias, mask, mask_bits, out,
                           row_begin, row_end, cols, (int32_t)has_bias, (int32_t)has_pre, P);
    return hipGetLastError();
}

// Enqueue the softmax of every call (all with the same row length).  Calls that can use a
// fixed-row-length kernel are grouped, up to kBatchMax per launch, while they agree on what
// the kernel instantiation fixes (bias or not, post step, packed or 32-bit arithmetic); the
// rows a slab decomposition leaves over, and calls it cannot serve, go to the generic kernel.
bool softmax_rows_compiled(int32_t cols)
{
#define IPTQ_IS_ROWS_SHAPE(COLS, K) if (cols == COLS) return true;
    IPTQ_ROWS_SHAPES(IPTQ_IS_ROWS_SHAPE)
#undef IPTQ_IS_ROWS_SHAPE
    return false;
}

hipError_t softmax_dispatch(const SoftmaxCall *calls, int n_calls, int32_t cols, hipStream_t stream)
{
    // A single call of a few thousand rows is one generation of wavefronts whatever the kernel:
    // its duration is one wavefront's chain of load, arithmetic and store, and one wavefront per
    // row has the shortest (kernel-trace durations, 591 / 2364 / 4728 rows of 197 scores: 3.6 /
    // 4.1 / 4.9 us against 5.5 / 5.3 / 4.9 us with the slab kernel; 392 to 3136 rows of 49 with a
    // table: 3.5-4.2 against 5.3-4.7 us; the slab kernels win from about 4000 rows on).
    constexpr int64_t kTinyRows = 3072;
    // (a per-window mask and the second-degree exponential exist in the compiled-row-length and
    // the three-pass kernels only)
    auto slab_only = [](const SoftmaxCall &c) {
        return c.mask != nullptr || c.mask_bits != nullptr || c.P.variant == 2;
    };
    if (n_calls == 1 && calls[0].algo == IPTQ_ALGO_AUTO && calls[0].rows <= kTinyRows && !slab_only(calls[0])) {
        int64_t served = 0;
        const hipError_t e = softmax_wide_launch(calls[0], cols, post_mode_of(calls[0].P, calls[0].out_bits),
                                                 &served, stream);
        if (e != hipSuccess) return e;
        if (served == calls[0].rows) return hipSuccess;      // every row or none
    }
    int rpw = 0;                                      // rows per wavefront of the compiled row length
    hipError_t (*launch)(const SoftmaxBatch &, unsigned, bool, int, bool, int, int, hipStream_t) = nullptr;
#define IPTQ_PICK_ROWS_SHAPE(COLS, K)                                                             \
    if (cols == COLS) { rpw = 64 / K; launch = launch_softmax_rows<COLS, K>; }
    IPTQ_ROWS_SHAPES(IPTQ_PICK_ROWS_SHAPE)
    int64_t total_rows = 0;
    for (int i = 0; i < n_calls; ++i) total_rows += calls[i].rows;
    if (total_rows * cols <= kRowsAltMaxElements) {   // a short launch: more lanes per row
        IPTQ_ROWS_SHAPES_ALT(IPTQ_PICK_ROWS_SHAPE)
    }
#undef IPTQ_PICK_ROWS_SHAPE
    SoftmaxBatch B;
    B.n_items = 0;
    unsigned total_wgs = 0;
    bool g_bias = false, g_fold = false;
    int g_mask = 0, g_pm = 0, g_mode = 0;             // g_mask: 0 none, 1 int32 table, 2 one bit per key
    hipError_t err = hipSuccess;
    auto flush = [&]() {
        if (B.n_items == 0 || err != hipSuccess) return;
        err = launch(B, total_wgs, g_bias, g_mask, g_fold, g_mode, g_pm, stream);
        g_fold = false;
        B.n_items = 0;
        total_wgs = 0;
    };
    int64_t done[kBatchMax];
    for (int base = 0; base < n_calls; base += kBatchMax) {
        const int cnt = n_calls - base < kBatchMax ? n_calls - base : kBatchMax;
        for (int i = 0; i < cnt; ++i) {
            const SoftmaxCall &c = calls[base + i];
            done[i] = 0;
            const bool has_bias = c.bias != nullptr;
            // the slab kernels load and store 16 bytes at any element address: views that start
            // off the 16-byte grid need nothing but their natural alignment
            const bool aligned =
                ((reinterpret_cast<uintptr_t>(c.scores) | reinterpret_cast<uintptr_t>(c.bias)) & 3) == 0;
            // the fused bias wraps at most once per slab, and its byte offsets are 32-bit
            const bool bias_ok = !has_bias || ((int64_t)c.P.bias_period_rows * cols >= 4 &&
                                       (int64_t)c.P.bias_period_rows * cols < ((int64_t)1 << 30) &&
                                               c.P.bias_period_rows >= rpw);
            const bool slab_algo = c.algo == IPTQ_ALGO_AUTO || c.algo == IPTQ_ALGO_SLAB;
            const int has_mask = c.mask != nullptr ? 1 : (c.mask_bits != nullptr ? 2 : 0);
            // the mask is compiled in beside a bias, for window sizes whose slab has no more rows
            // than a window has queries (49 and 144 tokens, in either form of the mask)
            bool mask_ok = true;
            if (has_mask == 1)
                mask_ok = has_bias && rows_mask_compiled(cols) && rpw <= cols &&
                          (reinterpret_cast<uintptr_t>(c.mask) & 3) == 0;
            else if (has_mask == 2)
                mask_ok = has_bias && rows_maskbits_compiled(cols) &&
                          (reinterpret_cast<uintptr_t>(c.mask_bits) & 7) == 0;
            if (rpw == 0 || !slab_algo || !aligned || !bias_ok || !mask_ok) continue;
            const int64_t n_slabs = (c.rows + rpw - 1) / rpw;    // a partial last slab is served too
            if (n_slabs == 0) continue;
            const int pm = post_mode_of(c.P, c.out_bits);
            const int mode = c.P.mode16;
            const bool compatible = B.n_items == 0 || (has_bias == g_bias && has_mask == g_mask && pm == g_pm &&
                                                       (mode == 0) == (g_mode == 0));
            if (!compatible || B.n_items == kBatchMax) flush();
            if (B.n_items == 0) { g_bias = has_bias; g_mask = has_mask; g_pm = pm; g_mode = mode; }
            else if (mode > g_mode) g_mode = mode;       // 2 covers 1: items with t16 == 0 shift by 0
            if (c.P.pre_rowconst != 0) g_fold = true;
            SoftmaxItem &it = B.item[B.n_items++];
            it.scores = c.scores; it.bias = c.bias; it.mask = c.mask; it.mask_bits = c.mask_bits; it.out = c.out;
            it.n_slabs = n_slabs; it.first_wg = total_wgs; it.P = c.P;
            it.tail_rows = (int32_t)(c.rows % rpw);
            it.share_q = 0; it.share_magic = 0; it.share_sh = 0;
            int64_t n_wgs = (n_slabs + kRowsWpb - 1) / kRowsWpb;
            if (has_bias) {
                // rows after which the tables repeat: the bias period, or with a mask the least
                // common multiple of both periods
                int64_t period = c.P.bias_period_rows;
                if (has_mask != 0) {
                    int64_t a = period, b = c.P.mask_period_rows;
                    while (b != 0) { const int64_t t = a % b; a = b; b = t; }
                    period = period / a * c.P.mask_period_rows;
                }
                int64_t a = period, b = rpw;
                while (b != 0) { const int64_t t = a % b; a = b; b = t; }      // a = gcd
                const int64_t q = period / a;
                if (q >= 2 && q < 65536 && q * kRowsWpb <= n_slabs &&
                    make_magic_u32((uint32_t)q, 31, &it.share_magic, &it.share_sh)) {
                    it.share_q = (uint32_t)q;
                    n_wgs = (n_slabs + kRowsWpb * q - 1) / (kRowsWpb * q) * q;
                }
            }
            total_wgs += (unsigned)n_wgs;
            done[i] = c.rows;
        }
        flush();
        for (int i = 0; i < cnt && err == hipSuccess; ++i) {
            const SoftmaxCall &c = calls[base + i];
            const bool has_pre = !(c.P.pre_m == 1 && c.P.pre_s == 0);
            // a call no compiled row length served goes to the run-time-row-length kernels
            if (done[i] == 0 && !slab_only(c) && (c.algo == IPTQ_ALGO_AUTO || c.algo == IPTQ_ALGO_DYNAMIC || c.algo == IPTQ_ALGO_SLAB)) {
                err = softmax_rowsdyn_launch(c, cols, post_mode_of(c.P, c.out_bits), &done[i], stream);
                if (err != hipSuccess) break;
            }
            if (done[i] == 0 && !slab_only(c) && (c.algo == IPTQ_ALGO_AUTO || c.algo == IPTQ_ALGO_WIDE)) {
                err = softmax_wide_launch(c, cols, post_mode_of(c.P, c.out_bits), &done[i], stream);
                if (err != hipSuccess) break;
            }
            if (done[i] == 0 && !slab_only(c) && (c.algo == IPTQ_ALGO_AUTO || c.algo == IPTQ_ALGO_WIDE)) {
                err = softmax_wgrow_launch(c, cols, post_mode_of(c.P, c.out_bits), &done[i], stream);
                if (err != hipSuccess) break;
            }
            err = launch_generic(c.scores, c.bias, c.mask, c.mask_bits, c.out, done[i], c.rows, cols, c.bias != nullptr,
                                 has_pre, c.P, stream);
        }
        if (err != hipSuccess) return err;
    }
    return err;
}

}  // namespace iptq
