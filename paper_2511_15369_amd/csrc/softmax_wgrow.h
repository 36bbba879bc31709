// Integer softmax (Section 4.4, Eq. 6-15) for very long rows: one workgroup of WAVES
// wavefronts per row, the row held in the workgroup's registers, read from HBM once.  The
// layout is that of the one-wavefront-per-row kernel (softmax_wide.h) with 64 * WAVES lanes:
// thread t of pass s owns the 16-byte block s * 64 * WAVES + t of the aligned block range that
// covers the row.  The row maximum and the row sum cross wavefronts through LDS and a
// workgroup barrier each.  Rows of up to 256 * WAVES * SLOTS - 3 scores.
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

template <int WAVES, int SLOTS, int MODE, int POSTMODE>
__global__ void __launch_bounds__(64 * WAVES)
softmax_wgrow_kernel(WideArgs A)
{
    constexpr int T = 64 * WAVES;                     // lanes that share the row
    __shared__ uint8_t lut[POSTMODE == PM_GENERAL ? kPostLutBytes : 4];
    __shared__ int32_t part_max[WAVES];
    __shared__ uint32_t part_sum[WAVES];
    const SoftmaxDev P = A.P;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wv = tid >> 6;
    const int64_t row = blockIdx.x;                   // grid == rows: every thread reaches every barrier

    if (POSTMODE == PM_GENERAL) {                     // visible to all after the barrier of the maximum
        const int p_max = 1 << (P.m_bits - P.p_shift);
        for (int p = tid; p <= p_max; p += T) lut[p] = (uint8_t)post_dev<PM_GENERAL>((uint32_t)p, P);
    }

    const int cols = A.cols;
    const int64_t e0 = row * cols;                    // the row's first element in the tensor
    const int phi = (int)(e0 & 3);                    // its offset inside its 16-byte block
    const int nb = (phi + cols + 3) >> 2;             // blocks the row touches
    const int n_used = (nb + T - 1) / T;              // passes that hold row data, <= SLOTS (host)
    const i32x4 *src = reinterpret_cast<const i32x4 *>(A.scores) + (e0 >> 2);

    // ---- the row's blocks; every load issued before the first use, threads beyond the last
    // block load it again (no divergent branch around a load)
    i32x4 v[SLOTS];
#pragma unroll
    for (int s = 0; s < SLOTS; ++s)
        if (s < n_used) v[s] = stream_load(src + min(s * T + tid, nb - 1));
    if (A.bias != nullptr) {
        const int64_t eb = (int64_t)row_mod_period((uint32_t)row, P) * cols;
        const i32x4 *bsrc = reinterpret_cast<const i32x4 *>(A.bias) + (eb >> 2);
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            if (s < n_used) {
                const i32x4 bv = bsrc[min(s * T + tid, nb - 1)];
                v[s].x = v[s].x == kI32Min ? kI32Min : sat_add_i32(v[s].x, bv.x);
                v[s].y = v[s].y == kI32Min ? kI32Min : sat_add_i32(v[s].y, bv.y);
                v[s].z = v[s].z == kI32Min ? kI32Min : sat_add_i32(v[s].z, bv.z);
                v[s].w = v[s].w == kI32Min ? kI32Min : sat_add_i32(v[s].w, bv.w);
            }
        }
    }

    // ---- elements outside the row become "minus infinity"
    int32_t x[SLOTS][4];
#pragma unroll
    for (int s = 0; s < SLOTS; ++s) {
        if (s >= n_used) {
            x[s][0] = x[s][1] = x[s][2] = x[s][3] = kI32Min;
            continue;
        }
        x[s][0] = v[s].x; x[s][1] = v[s].y; x[s][2] = v[s].z; x[s][3] = v[s].w;
        if (s == 0 || 4 * (s * T + T - 1) + 3 >= cols) {
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
        for (int s = 0; s < SLOTS; ++s) {
            if (s >= n_used) continue;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int32_t r = pre_requant_narrow(x[s][e], pre_mul, pre_rnd, pre_sh2);
                x[s][e] = x[s][e] == kI32Min ? kI32Min : r;
            }
        }
    } else if (P.pre_mode == 2) {
        const int32_t pre_m = P.pre_m, pre_s = P.pre_s;
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            if (s >= n_used) continue;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int32_t r = pre_requant_dev(x[s][e], pre_m, pre_s);
                x[s][e] = x[s][e] == kI32Min ? kI32Min : r;
            }
        }
    }

    // ---- Eq. 6: row maximum over the workgroup
    int32_t mx = kI32Min;
#pragma unroll
    for (int s = 0; s < SLOTS; ++s) {
        if (s >= n_used) continue;
#pragma unroll
        for (int e = 0; e < 4; ++e) mx = max(mx, x[s][e]);
    }
    mx = group_max_i32<64>(mx);
    if (lane == 0) part_max[wv] = mx;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < WAVES; ++i) mx = max(mx, part_max[i]);

    const int32_t D = P.d_clamp;
    const bool low_row = mx < kI32Min + D;            // workgroup-uniform; see softmax_rows_kernel
    const int32_t lower = low_row ? kI32Min : mx - D;
    uint32_t w[SLOTS];                                // four output bytes per block
    const WorkgroupSum<WAVES> wg_sum{part_sum, wv, lane};
    if (P.variant == 0)
        softmax_slab_math<64, SLOTS, MODE, 0, POSTMODE, true, WorkgroupSum<WAVES>>(x, w, mx, lower, low_row, lut, P, n_used, wg_sum);
    else
        softmax_slab_math<64, SLOTS, MODE, 1, POSTMODE, true, WorkgroupSum<WAVES>>(x, w, mx, lower, low_row, lut, P, n_used, wg_sum);

    // ---- write back: whole blocks as dwords, the two shared edge blocks byte by byte
    uint8_t *dst8 = A.out + (e0 - phi);
#pragma unroll
    for (int s = 0; s < SLOTS; ++s) {
        if (s >= n_used) continue;
        const int b = s * T + tid;
        const int c0 = 4 * b - phi;
        if (s != 0 && 4 * (s * T + T - 1) + 3 < cols) {
            stream_store(w[s], reinterpret_cast<uint32_t *>(dst8) + b);
        } else if (b < nb) {
            if (c0 >= 0 && c0 + 3 < cols) {
                stream_store(w[s], reinterpret_cast<uint32_t *>(dst8) + b);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if ((unsigned)(c0 + e) < (unsigned)cols) dst8[4 * b + e] = (uint8_t)(w[s] >> (8 * e));
            }
        }
    }
}

template <int WAVES, int SLOTS>
static void wgrow_launch_ws(const WideArgs &A, int mode, int post_mode, dim3 grid, hipStream_t stream)
{
#define IPTQ_WGROW_LAUNCH(MODE, PM)                                                               \
    hipLaunchKernelGGL((softmax_wgrow_kernel<WAVES, SLOTS, MODE, PM>), grid, dim3(64 * WAVES), 0, stream, A)
    if (mode == 0) {
        if (post_mode == PM_NONE) IPTQ_WGROW_LAUNCH(0, PM_NONE);
        else if (post_mode == PM_CLAMP127) IPTQ_WGROW_LAUNCH(0, PM_CLAMP127);
        else IPTQ_WGROW_LAUNCH(0, PM_GENERAL);
    } else {                                          // 2 covers 1: t16 == 0 shifts by 0
        if (post_mode == PM_NONE) IPTQ_WGROW_LAUNCH(2, PM_NONE);
        else if (post_mode == PM_CLAMP127) IPTQ_WGROW_LAUNCH(2, PM_CLAMP127);
        else IPTQ_WGROW_LAUNCH(2, PM_GENERAL);
    }
#undef IPTQ_WGROW_LAUNCH
}

// one translation unit per layout (softmax_wgrow_w<WAVES>_s<SLOTS>.hip)
void wgrow_launch_w4_s13(const WideArgs &A, int mode, int post_mode, dim3 grid, hipStream_t stream);
void wgrow_launch_w4_s20(const WideArgs &A, int mode, int post_mode, dim3 grid, hipStream_t stream);
void wgrow_launch_w8_s16(const WideArgs &A, int mode, int post_mode, dim3 grid, hipStream_t stream);
void wgrow_launch_w8_s20(const WideArgs &A, int mode, int post_mode, dim3 grid, hipStream_t stream);

}  // namespace iptq
