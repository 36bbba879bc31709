// Integer softmax for any row length that fits LDS (Section 4.4, Eq. 6-15): the same slab
// scheme as the fixed-row-length kernel, with the row length and the number of lanes per
// row as run-time values.  A wavefront owns R = 64 / L whole rows (L lanes per row, a power
// of two chosen on the host so that R * cols is a multiple of 4 and the slab starts on a
// 16-byte boundary).  The slab is copied flat into LDS (bias and pre-requantization applied
// on the way), and three passes run over LDS instead of registers:
//   1. row maximum;
//   2. exponentials, written back over the scores, and the row sum;
//   3. probabilities, assembled as bytes in a second LDS area, then stored flat.
// HBM is read once and written once.  Row-length-specific unrolling is what the fixed
// kernels add on top of this.
#include <hip/hip_runtime.h>

#include "device_common.h"
#include "kernels.h"
#include "plan.h"
#include "softmax_rows.h"

namespace iptq {

struct FlexArgs {
    const int32_t *scores;
    const int32_t *bias;
    uint8_t *out;
    int64_t n_slabs;      // the last one may be partial
    int32_t tail_rows;    // rows of the last slab if it is partial, else 0
    int32_t cols;
    int32_t log2_lanes;   // lanes per row = 1 << log2_lanes
    int32_t post_mode;    // PM_*
    int32_t has_pre;
    int32_t wave_lds;     // LDS bytes per wavefront (multiple of 16)
    SoftmaxDev P;
};

IPTQ_DEV int32_t group_max_rt(int32_t v, int log2_lanes)
{
    if (log2_lanes >= 1) v = max(v, dpp_i32<0xB1>(v));
    if (log2_lanes >= 2) v = max(v, dpp_i32<0x4E>(v));
    if (log2_lanes >= 3) v = max(v, dpp_i32<0x141>(v));
    if (log2_lanes >= 4) v = max(v, dpp_i32<0x140>(v));
    if (log2_lanes >= 5) v = max(v, __shfl_xor(v, 16));
    if (log2_lanes >= 6) v = max(v, __shfl_xor(v, 32));
    return v;
}

IPTQ_DEV uint32_t group_sum_rt(uint32_t v, int log2_lanes)
{
    if (log2_lanes >= 1) v += (uint32_t)dpp_i32<0xB1>((int32_t)v);
    if (log2_lanes >= 2) v += (uint32_t)dpp_i32<0x4E>((int32_t)v);
    if (log2_lanes >= 3) v += (uint32_t)dpp_i32<0x141>((int32_t)v);
    if (log2_lanes >= 4) v += (uint32_t)dpp_i32<0x140>((int32_t)v);
    if (log2_lanes >= 5) v += (uint32_t)__shfl_xor((int32_t)v, 16);
    if (log2_lanes >= 6) v += (uint32_t)__shfl_xor((int32_t)v, 32);
    return v;
}

// elements of block b that lie outside the row become "minus infinity"
IPTQ_DEV i32x4 mask_block(i32x4 v, int c0, int cols)
{
    if (c0 < 0 || c0 + 3 >= cols) {
        if ((unsigned)(c0 + 0) >= (unsigned)cols) v.x = kI32Min;
        if ((unsigned)(c0 + 1) >= (unsigned)cols) v.y = kI32Min;
        if ((unsigned)(c0 + 2) >= (unsigned)cols) v.z = kI32Min;
        if ((unsigned)(c0 + 3) >= (unsigned)cols) v.w = kI32Min;
    }
    return v;
}

// pass 2 for one lane: exponentials of its blocks, written back in place; returns its sum
template <bool PACKED, int VARIANT>
IPTQ_DEV uint32_t flex_exp_pass(uint8_t *lds, int b_r, int phi, int nb, int j, int lanes, int cols,
                                int32_t mx, int32_t lower, const SoftmaxDev &P)
{
    i32x4 *lds4 = reinterpret_cast<i32x4 *>(lds);
    uint32_t *lds32 = reinterpret_cast<uint32_t *>(lds);
    uint32_t sum = 0;
#pragma unroll 2
    for (int b = j; b < nb; b += lanes) {
        const int c0 = 4 * b - phi;
        const i32x4 v = mask_block(lds4[b_r + b], c0, cols);
        u32x4 q;
        if (PACKED) {
            const u16x2 e01 = bit_exp_pair<VARIANT, true>(v.x, v.y, mx, P);
            const u16x2 e23 = bit_exp_pair<VARIANT, true>(v.z, v.w, mx, P);
            sum = __builtin_amdgcn_udot2(e01, (u16x2){1, 1}, sum, false);
            sum = __builtin_amdgcn_udot2(e23, (u16x2){1, 1}, sum, false);
            q = (u32x4){e01.x, e01.y, e23.x, e23.y};
        } else {
            q.x = bit_exp_dev<VARIANT, true>(v.x, lower, mx, P);
            q.y = bit_exp_dev<VARIANT, true>(v.y, lower, mx, P);
            q.z = bit_exp_dev<VARIANT, true>(v.z, lower, mx, P);
            q.w = bit_exp_dev<VARIANT, true>(v.w, lower, mx, P);
            sum += q.x + q.y + q.z + q.w;
        }
        if (c0 >= 0 && c0 + 3 < cols) {
            reinterpret_cast<u32x4 *>(lds)[b_r + b] = q;
        } else {                                  // a block shared with a neighbour row
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if ((unsigned)(c0 + e) < (unsigned)cols) lds32[4 * (b_r + b) + e] = q[e];
        }
    }
    return sum;
}

template <int MODE>   // 0: 32-bit lanes, 2: packed 16-bit lanes (with the n << t16 step)
__global__ void __launch_bounds__(256)
softmax_flex_kernel(FlexArgs A)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t flex_lds[];
    const SoftmaxDev &P = A.P;
    const int lane = threadIdx.x & 63;
    const int wv = threadIdx.x >> 6;
    const int64_t slab = (int64_t)blockIdx.x * (blockDim.x >> 6) + wv;
    if (slab >= A.n_slabs) return;                    // no workgroup barrier below

    const int cols = A.cols;
    const int log2l = A.log2_lanes;
    const int lanes = 1 << log2l;
    const int rpw = 64 >> log2l;
    const int slab_el = rpw * cols;                   // multiple of 4 (host)
    uint8_t *lds = flex_lds + wv * A.wave_lds;
    uint8_t *lds_out = lds + slab_el * 4;             // byte assembly area, 16-byte aligned
    const int32_t *src1 = A.scores + slab * slab_el;
    const i32x4 *src = reinterpret_cast<const i32x4 *>(src1);
    // a partial last slab reads and writes nothing beyond its last valid element; its
    // surplus rows are zero-filled, computed and never stored
    const bool partial = A.tail_rows != 0 && slab == A.n_slabs - 1;
    const int valid_el = (partial ? A.tail_rows : rpw) * cols;

    // ---- flat copy into LDS; bias and pre-requantization on the way
    {
        i32x4 *lds4 = reinterpret_cast<i32x4 *>(lds);
        const bool has_bias = A.bias != nullptr;
        uint32_t boff = 0;
        if (has_bias) boff = row_mod_period((uint32_t)(slab * rpw), P) * (uint32_t)cols;
        const uint32_t pe = (uint32_t)P.bias_period_rows * (uint32_t)cols;
        for (int idx = lane; idx < (slab_el >> 2); idx += 64) {
            i32x4 v;
            if (4 * idx + 3 < valid_el) {
                v = stream_load(src + idx);
            } else {
                v = (i32x4){0, 0, 0, 0};
                if (4 * idx < valid_el) v.x = src1[4 * idx];
                if (4 * idx + 1 < valid_el) v.y = src1[4 * idx + 1];
                if (4 * idx + 2 < valid_el) v.z = src1[4 * idx + 2];
            }
            if (has_bias) {
                uint32_t o = boff + 4u * (uint32_t)idx;
                if (o >= pe) o -= pe;
                const i32x4 bv = *reinterpret_cast<const i32x4 *>(A.bias + o);
                v.x = v.x == kI32Min ? v.x : sat_add_i32(v.x, bv.x);
                v.y = v.y == kI32Min ? v.y : sat_add_i32(v.y, bv.y);
                v.z = v.z == kI32Min ? v.z : sat_add_i32(v.z, bv.z);
                v.w = v.w == kI32Min ? v.w : sat_add_i32(v.w, bv.w);
            }
            if (A.has_pre) {
                v.x = v.x == kI32Min ? v.x : pre_requant_dev(v.x, P.pre_m, P.pre_s);
                v.y = v.y == kI32Min ? v.y : pre_requant_dev(v.y, P.pre_m, P.pre_s);
                v.z = v.z == kI32Min ? v.z : pre_requant_dev(v.z, P.pre_m, P.pre_s);
                v.w = v.w == kI32Min ? v.w : pre_requant_dev(v.w, P.pre_m, P.pre_s);
            }
            lds4[idx] = v;
        }
        wave_lds_fence();
    }

    const int lr = lane >> log2l;                     // row inside the slab
    const int j = lane & (lanes - 1);                 // lane inside the row
    const int e_r = lr * cols;                        // first element of the row in the slab
    const int b_r = e_r >> 2;                         // its 16-byte block
    const int phi = e_r & 3;                          // and its offset inside that block
    const int nb = (phi + cols + 3) >> 2;             // blocks the row touches
    const i32x4 *lds4 = reinterpret_cast<const i32x4 *>(lds);

    // ---- pass 1, Eq. 6: row maximum
    int32_t mx = kI32Min;
#pragma unroll 2
    for (int b = j; b < nb; b += lanes) {
        const i32x4 v = mask_block(lds4[b_r + b], 4 * b - phi, cols);
        mx = max(max(mx, max(v.x, v.y)), max(v.z, v.w));
    }
    mx = group_max_rt(mx, log2l);
    const int32_t D = P.d_clamp;
    const bool low_row = mx < kI32Min + D;
    const int32_t lower = low_row ? kI32Min : mx - D;
    const bool packed = MODE != 0 && __builtin_amdgcn_ballot_w64(low_row) == 0;

    // ---- pass 2: exponentials and row sum
    uint32_t sum;
    if (packed) {
        sum = P.variant == 0 ? flex_exp_pass<true, 0>(lds, b_r, phi, nb, j, lanes, cols, mx, lower, P)
                             : flex_exp_pass<true, 1>(lds, b_r, phi, nb, j, lanes, cols, mx, lower, P);
    } else {
        sum = P.variant == 0 ? flex_exp_pass<false, 0>(lds, b_r, phi, nb, j, lanes, cols, mx, lower, P)
                             : flex_exp_pass<false, 1>(lds, b_r, phi, nb, j, lanes, cols, mx, lower, P);
    }
    sum = group_sum_rt(sum, log2l);

    // ---- pass 3, Eq. 15: one reciprocal per row, probabilities into the byte area
    const uint32_t f = floor_pow2_div(P.m_bits, sum);
    const uint32_t f_top = P.p_shift <= 24 ? f << (24 - P.p_shift) : 0u;
    uint32_t *out32 = reinterpret_cast<uint32_t *>(lds_out);
#pragma unroll 2
    for (int b = j; b < nb; b += lanes) {
        const int c0 = 4 * b - phi;
        const u32x4 q = reinterpret_cast<const u32x4 *>(lds)[b_r + b];
        uint32_t w;
        if (A.post_mode == PM_NONE) w = normalise4<PM_NONE>(q.x, q.y, q.z, q.w, f, f_top, P);
        else if (A.post_mode == PM_CLAMP127) w = normalise4<PM_CLAMP127>(q.x, q.y, q.z, q.w, f, f_top, P);
        else w = normalise4<PM_GENERAL>(q.x, q.y, q.z, q.w, f, f_top, P);
        if (c0 >= 0 && c0 + 3 < cols) {
            out32[b_r + b] = w;
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if ((unsigned)(c0 + e) < (unsigned)cols) lds_out[4 * (b_r + b) + e] = (uint8_t)(w >> (8 * e));
        }
    }
    wave_lds_fence();

    // ---- flat store of the slab's bytes
    uint8_t *dst = A.out + slab * slab_el;
    if ((slab_el & 15) == 0) {
        const u32x4 *o4 = reinterpret_cast<const u32x4 *>(lds_out);
        for (int idx = lane; idx < (slab_el >> 4); idx += 64) {
            if (16 * idx + 15 < valid_el) {
                stream_store(o4[idx], reinterpret_cast<u32x4 *>(dst) + idx);
            } else {
#pragma unroll 1
                for (int b = 16 * idx; b < valid_el && b < 16 * idx + 16; ++b) dst[b] = lds_out[b];
            }
        }
    } else {
        for (int idx = lane; idx < (slab_el >> 2); idx += 64) {
            if (4 * idx + 3 < valid_el) {
                stream_store(out32[idx], reinterpret_cast<uint32_t *>(dst) + idx);
            } else {
#pragma unroll 1
                for (int b = 4 * idx; b < valid_el && b < 4 * idx + 4; ++b) dst[b] = lds_out[b];
            }
        }
    }
}

// Lanes per row for a row length.  The alignment rule bounds it (R * cols must be a multiple
// of 4).  The run-time loops are latency-bound, so what pays is many resident wavefronts
// (small slabs) as long as a wavefront still has enough elements to amortise its fixed work
// (staging, reductions, one reciprocal): take the largest lane count that keeps at least
// kFlexMinSlab elements per wavefront and does not idle more than 40 % of the lanes in the
// block loop; otherwise the allowed choice with the largest slab.  The slab must fit the LDS
// budget.  Returns false if no choice fits.
// LDS per wavefront may reach a whole workgroup's 64 KB (then a workgroup is one wavefront)
constexpr int64_t kFlexMaxWaveLds = 64 * 1024;
#ifndef IPTQ_FLEX_MIN_SLAB
#define IPTQ_FLEX_MIN_SLAB 768
#endif
bool flex_geometry(int32_t cols, int *log2_lanes, int *wave_lds)
{
    const int max_log2 = (cols % 4 == 0) ? 6 : ((cols % 2 == 0) ? 5 : 4);
    const int nb = (cols % 4 == 0) ? cols / 4 : (cols + 3 + 3) / 4;
    int best = -1, fallback = -1;
    for (int l2 = 0; l2 <= max_log2; ++l2) {
        const int lanes = 1 << l2, rpw = 64 >> l2;
        const int64_t bytes = ((int64_t)rpw * cols * 5 + 15) & ~(int64_t)15;
        if (bytes > kFlexMaxWaveLds) continue;
        if (fallback < 0) fallback = l2;              // fewest lanes that fit: the largest slab
        const int per_lane = (nb + lanes - 1) / lanes;
        const double util = (double)cols / (4.0 * per_lane * lanes);
        if (rpw * cols >= IPTQ_FLEX_MIN_SLAB && util >= 0.6) best = l2;
    }
    if (best < 0) best = fallback;
    if (best < 0) return false;
    *log2_lanes = best;
    *wave_lds = (int)((((int64_t)(64 >> best) * cols * 5) + 15) & ~(int64_t)15);
    return true;
}

// Every row of one call (a partial last slab included) if the call qualifies; returns the
// number of rows served through *done.
hipError_t softmax_flex_launch(const SoftmaxCall &c, int32_t cols, int post_mode, int64_t *done,
                               hipStream_t stream)
{
    *done = 0;
    int log2l = 0, wave_lds = 0;
    if (!flex_geometry(cols, &log2l, &wave_lds)) return hipSuccess;
    const int rpw = 64 >> log2l;
    const bool has_bias = c.bias != nullptr;
    const bool aligned = ((reinterpret_cast<uintptr_t>(c.scores) & 15) | (reinterpret_cast<uintptr_t>(c.out) & 15)) == 0;
    const bool bias_ok = !has_bias || ((reinterpret_cast<uintptr_t>(c.bias) & 15) == 0 &&
                                       ((int64_t)c.P.bias_period_rows * cols) % 4 == 0 &&
                                       (int64_t)c.P.bias_period_rows * cols < ((int64_t)1 << 31) &&
                                       c.P.bias_period_rows >= rpw);
    const int64_t n_slabs = (c.rows + rpw - 1) / rpw;
    if (!aligned || !bias_ok || n_slabs == 0) return hipSuccess;
    FlexArgs A;
    A.scores = c.scores; A.bias = c.bias; A.out = c.out; A.n_slabs = n_slabs; A.cols = cols;
    A.tail_rows = (int32_t)(c.rows % rpw);
    A.log2_lanes = log2l; A.post_mode = post_mode;
    A.has_pre = !(c.P.pre_m == 1 && c.P.pre_s == 0);
    A.wave_lds = wave_lds; A.P = c.P;
    int wpb = (int)(kFlexMaxWaveLds / wave_lds);      // wavefronts per workgroup: 1..4
    if (wpb > 4) wpb = 4;
    const dim3 grid((unsigned)((n_slabs + wpb - 1) / wpb)), block(64 * wpb);
    const size_t lds = (size_t)wave_lds * wpb;
    if (c.P.mode16 != 0 && post_mode != PM_GENERAL)
        hipLaunchKernelGGL(softmax_flex_kernel<2>, grid, block, lds, stream, A);
    else
        hipLaunchKernelGGL(softmax_flex_kernel<0>, grid, block, lds, stream, A);
    *done = c.rows;
    return hipGetLastError();
}

}  // namespace iptq
