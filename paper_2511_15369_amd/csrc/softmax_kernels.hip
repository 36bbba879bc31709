// Integer softmax for gfx950 (Section 4.4, Eq. 6-15): the any-row-length kernel and the
// dispatch between it and the fixed-row-length kernels of softmax_rows.h.
//   softmax_generic_kernel - run-time row length, one wavefront per row, three passes.
//                          Serves odd shapes, the tail rows of the fixed-length kernels and
//                          the fused pre-requantization.
#include <hip/hip_runtime.h>

#include "device_common.h"
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
                       uint8_t *__restrict__ out, int64_t row_begin, int64_t row_end, int32_t cols,
                       int32_t has_bias, int32_t has_pre, SoftmaxDev P)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = row_begin + (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= row_end) return;
    const int32_t *srow = scores + row * cols;
    const int32_t *brow = nullptr;
    if (has_bias) brow = bias + (int64_t)row_mod_period((uint32_t)row, P) * cols;

    auto fetch = [&](int c) -> int32_t {
        int32_t v = srow[c];
        if (has_bias && v != kI32Min) v = sat_add_i32(v, brow[c]);
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
// Host-side dispatch.

static int post_mode_of(const SoftmaxDev &P, int out_bits)
{
    const bool identity = P.post_m == 1 && P.post_s == 0 && P.post_zp == 0 && P.qmin <= 0;
    if (!identity) return PM_GENERAL;
    if (P.qmax >= (1 << (out_bits - 1))) return PM_NONE;
    return (P.qmax == 127 && out_bits == 8) ? PM_CLAMP127 : PM_GENERAL;
}

static hipError_t launch_generic(const int32_t *scores, const int32_t *bias, uint8_t *out,
                                 int64_t row_begin, int64_t row_end, int32_t cols, bool has_bias,
                                 bool has_pre, const SoftmaxDev &P, hipStream_t stream)
{
    const int64_t n = row_end - row_begin;
    if (n <= 0) return hipSuccess;
    const dim3 grid((unsigned)((n + 3) / 4)), block(256);
    if (P.variant == 0)
        hipLaunchKernelGGL(softmax_generic_kernel<0>, grid, block, 0, stream, scores, bias, out,
                           row_begin, row_end, cols, (int32_t)has_bias, (int32_t)has_pre, P);
    else
        hipLaunchKernelGGL(softmax_generic_kernel<1>, grid, block, 0, stream, scores, bias, out,
                           row_begin, row_end, cols, (int32_t)has_bias, (int32_t)has_pre, P);
    return hipGetLastError();
}

// Enqueue the softmax of rows [0, rows).  Returns a hipError_t.
hipError_t softmax_dispatch(const int32_t *scores, const int32_t *bias, uint8_t *out, int64_t rows,
                            int32_t cols, int out_bits, bool force_generic, const SoftmaxDev &P,
                            hipStream_t stream)
{
    const bool has_bias = bias != nullptr;
    const bool has_pre = !(P.pre_m == 1 && P.pre_s == 0);
    const bool aligned = ((reinterpret_cast<uintptr_t>(scores) | reinterpret_cast<uintptr_t>(out)) & 15) == 0;
    const int post_mode = post_mode_of(P, out_bits);
    int64_t done = 0;
    if (!force_generic && !has_pre && aligned) {
        // the fused bias needs 16-byte aligned bias blocks and at most one wrap per slab
        auto bias_ok = [&](int rpw) {
            if (!has_bias) return true;
            return (reinterpret_cast<uintptr_t>(bias) & 15) == 0 &&
                   ((int64_t)P.bias_period_rows * cols) % 4 == 0 && P.bias_period_rows >= rpw;
        };
        hipError_t err = hipSuccess;
        constexpr int rpw197 = 64 / IPTQ_K197, rpw49 = 64 / IPTQ_K49;
        if (cols == 197 && bias_ok(rpw197)) {
            const int64_t n_slabs = rows / rpw197;
            if (n_slabs > 0)
                err = launch_softmax_rows<197, IPTQ_K197>(scores, bias, out, n_slabs, P.mode16, post_mode, P, stream);
            done = n_slabs * rpw197;
        } else if (cols == 49 && bias_ok(rpw49)) {
            const int64_t n_slabs = rows / rpw49;
            if (n_slabs > 0)
                err = launch_softmax_rows<49, IPTQ_K49>(scores, bias, out, n_slabs, P.mode16, post_mode, P, stream);
            done = n_slabs * rpw49;
        }
        if (err != hipSuccess) return err;
    }
    return launch_generic(scores, bias, out, done, rows, cols, has_bias, has_pre, P, stream);
}

}  // namespace iptq
