// Integer softmax (Section 4.4, Eq. 6-15) for very long rows: one workgroup of WAVES
// wavefronts per row, the row held in the workgroup's registers, read from HBM once.  The
// layout is that of the one-wavefront-per-row kernel (softmax_wide.h) with T = 64 * WAVES
// lanes: thread t of pass s owns the 16-byte block s * T + t of the aligned block range that
// covers the row.  The row maximum and the row sum cross wavefronts through LDS and a
// workgroup barrier each.  SLOTS is exactly the number of passes a row of this length needs
// at its worst alignment (see softmax_wide.h for what that fixes): no branch depends on the
// row length.
#pragma once

#include <hip/hip_runtime.h>

#include "device_common.h"
#include "kernels.h"
#include "plan.h"
#include "softmax_rows.h"
#include "softmax_wide.h"

namespace iptq {

// Sum over every lane of the workgroup: 64 lanes through DPP and the permute network, then
// the per-wavefront partials through LDS.  Every thread of the workgroup must call it.
template <int WAVES>
struct WorkgroupSum {
    uint32_t *partial;   // WAVES words of LDS
    int wv, lane;
    IPTQ_DEV uint32_t operator()(uint32_t v) const
    {
        v = group_sum_u32<64>(v);
        if (lane == 0) partial[wv] = v;
        __syncthreads();
        uint32_t t = 0;
#pragma unroll
        for (int i = 0; i < WAVES; ++i) t += partial[i];
        return t;
    }
};

template <int WAVES, int SLOTS, int MODE>
__global__ void __launch_bounds__(64 * WAVES)
softmax_wgrow_kernel(WideArgs A)
{
    constexpr int T = 64 * WAVES;                     // lanes that share the row
    __shared__ uint8_t lut[kPostLutBytes];
    __shared__ int32_t part_max[WAVES];
    __shared__ uint32_t part_sum[WAVES];
    touch_kernel_arguments<sizeof(WideArgs)>();
    const SoftmaxDev P = A.P;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wv = tid >> 6;
    const int64_t row = blockIdx.x;                   // grid == rows: every thread reaches every barrier

    const int post_mode = A.post_mode;
    if (post_mode == PM_GENERAL) {                    // visible to all after the barrier of the maximum
        const int p_max = 1 << (P.m_bits - P.p_shift);
        for (int p = tid; p <= p_max; p += T) lut[p] = (uint8_t)post_dev<PM_GENERAL>((uint32_t)p, P);
    }

    const int cols = A.cols;
    const int64_t e0 = row * cols + A.base_off;       // the row's first element on the 16-byte grid
    const int phi = (int)(e0 & 3);                    // its offset inside its 16-byte block
    const int nb = (phi + cols + 3) >> 2;             // blocks the row touches
    const i32x4 *src = reinterpret_cast<const i32x4 *>(A.scores) + (e0 >> 2);
    // the last row of a tensor that ends off the 16-byte grid: its final block is loaded
    // element by element below (workgroup-uniform case)
    const bool cut = A.cut_el != 0 && row == A.rows - 1;
    const int nb_whole = cut ? nb - 1 : nb;           // blocks that can be loaded whole, >= 1
    auto block_of = [&](int s, int n) {               // threads beyond block n - 1 load it again
        const int b = s * T + tid;
        return s >= SLOTS - 2 ? min(b, n - 1) : b;
    };
    auto edge_slot = [](int s) { return s == 0 || s >= SLOTS - 2; };

    // ---- the row's blocks; every load issued before the first use, none behind a branch
    i32x4 v[SLOTS];
#pragma unroll
    for (int s = 0; s < SLOTS; ++s) v[s] = stream_load(src + block_of(s, nb_whole));
    if (cut) {
        const int32_t *last = reinterpret_cast<const int32_t *>(src + (nb - 1));
#pragma unroll
        for (int s = SLOTS >= 2 ? SLOTS - 2 : 0; s < SLOTS; ++s) {
            if (s * T + tid == nb - 1) {              // elements beyond cut_el are masked below
                v[s].x = last[0];
                if (A.cut_el > 1) v[s].y = last[1];
                if (A.cut_el > 2) v[s].z = last[2];
            }
        }
    }
    if (A.bias != nullptr) {
        const int64_t eb = (int64_t)row_mod_period((uint32_t)row, P) * cols;
        const i32x4 *bsrc = reinterpret_cast<const i32x4 *>(A.bias) + (eb >> 2);
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            const i32x4 bv = bsrc[block_of(s, nb)];
            v[s] = add_table_chunk(v[s], bv);
        }
    }

    // ---- elements outside the row become "minus infinity"
    int32_t x[SLOTS][4];
#pragma unroll
    for (int s = 0; s < SLOTS; ++s) {
        x[s][0] = v[s].x; x[s][1] = v[s].y; x[s][2] = v[s].z; x[s][3] = v[s].w;
        if (edge_slot(s)) {
            const int c0 = 4 * (s * T + tid) - phi;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if ((unsigned)(c0 + e) >= (unsigned)cols) x[s][e] = kI32Min;
        }
    }

    // ---- fused requantization of the scores (after the bias, before the maximum)
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
    } else if (P.pre_mode == 2) {
        const int32_t pre_m = P.pre_m, pre_s = P.pre_s;
#pragma unroll
        for (int s = 0; s < SLOTS; ++s)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int32_t r = pre_requant_dev(x[s][e], pre_m, pre_s);
                x[s][e] = x[s][e] == kI32Min ? kI32Min : r;
            }
    }

    // ---- Eq. 6: row maximum over the workgroup
    int32_t mx = kI32Min;
#pragma unroll
    for (int s = 0; s < SLOTS; ++s)
#pragma unroll
        for (int e = 0; e < 4; ++e) mx = max(mx, x[s][e]);
    mx = group_max_i32<64>(mx);
    if (lane == 0) part_max[wv] = mx;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < WAVES; ++i) mx = max(mx, part_max[i]);

    const int32_t D = P.d_clamp;
    const bool low_row = mx < kI32Min + D;            // workgroup-uniform; see softmax_rows_kernel
    const int32_t lower = low_row ? kI32Min : mx - D;
    uint32_t w[SLOTS];                                // four probabilities per block, one per byte
    const WorkgroupSum<WAVES> wg_sum{part_sum, wv, lane};
    if (P.variant == 0)
        softmax_slab_math<64, SLOTS, MODE, 0, PM_NONE, WorkgroupSum<WAVES>>(x, w, mx, lower, low_row, lut, P, wg_sum);
    else
        softmax_slab_math<64, SLOTS, MODE, 1, PM_NONE, WorkgroupSum<WAVES>>(x, w, mx, lower, low_row, lut, P, wg_sum);

    // ---- post step on the packed bytes (a probability is at most 128)
    if (post_mode == PM_CLAMP127) {
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) w[s] = clamp127_bytes(w[s]);
    } else if (post_mode == PM_GENERAL) {
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) w[s] = post_lut_gather(lut, w[s]);
    } else if (P.post_xor != 0) {                     // signed output around the zero-point -128
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) w[s] ^= P.post_xor;
    }

    // ---- write back: whole blocks as dwords, the two shared edge blocks byte by byte
    uint8_t *dst8 = A.out + (e0 - phi);
#pragma unroll
    for (int s = 0; s < SLOTS; ++s) {
        const int b = s * T + tid;
        const int c0 = 4 * b - phi;
        if (!edge_slot(s)) {                          // every thread's block lies inside the row
            stream_store_bytes4(w[s], dst8 + 4 * b);
        } else if (b < nb) {
            if (c0 >= 0 && c0 + 3 < cols) {
                stream_store_bytes4(w[s], dst8 + 4 * b);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if ((unsigned)(c0 + e) < (unsigned)cols) dst8[4 * b + e] = (uint8_t)(w[s] >> (8 * e));
            }
        }
    }
}

// mode: SoftmaxDev::mode16 (2 covers 1: t16 == 0 shifts by 0)
template <int WAVES, int SLOTS>
static void wgrow_launch_ws(const WideArgs &A, int mode, dim3 grid, hipStream_t stream)
{
    if (mode == 0) hipLaunchKernelGGL((softmax_wgrow_kernel<WAVES, SLOTS, 0>), grid, dim3(64 * WAVES), 0, stream, A);
    else hipLaunchKernelGGL((softmax_wgrow_kernel<WAVES, SLOTS, 2>), grid, dim3(64 * WAVES), 0, stream, A);
}

// one translation unit per workgroup size and group of pass counts; each returns false for a
// count it does not hold
bool wgrow_launch_w4_lo(const WideArgs &A, int passes, int mode, dim3 grid, hipStream_t stream);
bool wgrow_launch_w4_hi(const WideArgs &A, int passes, int mode, dim3 grid, hipStream_t stream);
bool wgrow_launch_w8_lo(const WideArgs &A, int passes, int mode, dim3 grid, hipStream_t stream);
bool wgrow_launch_w8_hi(const WideArgs &A, int passes, int mode, dim3 grid, hipStream_t stream);
bool wgrow_launch_w16(const WideArgs &A, int passes, int mode, dim3 grid, hipStream_t stream);

#define IPTQ_WGROW_CASE(W, S)                                                                     \
    case S: wgrow_launch_ws<W, S>(A, mode, grid, stream); return true;

}  // namespace iptq
