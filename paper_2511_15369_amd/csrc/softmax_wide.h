// Integer softmax (Section 4.4, Eq. 6-15) for long rows: one wavefront per row, the row
// held in registers, no LDS staging.  All 64 lanes share the row: lane l of pass s owns the
// 16-byte block s * 64 + l of the aligned block range that covers the row, so a pass is one
// fully coalesced 1 KiB load.  A row that does not start on a 16-byte boundary shares its first
// and last block with its neighbours: their elements are masked on the way in and those
// blocks are written back with byte stores, every other block with one dword store.  The
// arithmetic is the slab kernels' (softmax_slab_math with 64 lanes per row).  Rows of up to
// 256 * SLOTS - 3 scores.
#pragma once

#include <hip/hip_runtime.h>

#include "device_common.h"
#include "kernels.h"
#include "plan.h"
#include "softmax_rows.h"

namespace iptq {

struct WideArgs {
    const int32_t *scores;   // 16-byte aligned
    const int32_t *bias;     // NULL or 16-byte aligned, period * cols a multiple of 4
    uint8_t *out;            // 4-byte aligned
    int64_t rows;            // rows served by this launch (the host keeps a last row whose final
                             // block would reach beyond the tensor out of it)
    int32_t cols;
    SoftmaxDev P;
};

template <int SLOTS, int MODE, int POSTMODE>
__global__ void __launch_bounds__(256)
softmax_wide_kernel(WideArgs A)
{
    __shared__ uint8_t lut_all[4][POSTMODE == PM_GENERAL ? kPostLutBytes : 4];
    const SoftmaxDev P = A.P;
    const int lane = threadIdx.x & 63;
    const int wv = threadIdx.x >> 6;
    const int64_t row = (int64_t)blockIdx.x * 4 + wv;
    if (row >= A.rows) return;                        // no workgroup barrier below

    uint8_t *lut = lut_all[wv];
    if (POSTMODE == PM_GENERAL) {
        const int p_max = 1 << (P.m_bits - P.p_shift);
        for (int p = lane; p <= p_max; p += 64) lut[p] = (uint8_t)post_dev<PM_GENERAL>((uint32_t)p, P);
        wave_lds_fence();
    }

    const int cols = A.cols;
    const int64_t e0 = row * cols;                    // the row's first element in the tensor
    const int phi = (int)(e0 & 3);                    // its offset inside its 16-byte block
    const int nb = (phi + cols + 3) >> 2;             // blocks the row touches (wavefront-uniform)
    const int n_used = (nb + 63) >> 6;                // passes that hold row data, <= SLOTS (host)
    const i32x4 *src = reinterpret_cast<const i32x4 *>(A.scores) + (e0 >> 2);

    // ---- the row's blocks; every load is issued before the first use, lanes beyond the last
    // block load it again (no lane-divergent branch around a load)
    i32x4 v[SLOTS];
#pragma unroll
    for (int s = 0; s < SLOTS; ++s)
        if (s < n_used) v[s] = stream_load(src + min(s * 64 + lane, nb - 1));
    if (A.bias != nullptr) {
        // the bias row starts at the same offset inside a block (period * cols % 4 == 0)
        const int64_t eb = (int64_t)row_mod_period((uint32_t)row, P) * cols;
        const i32x4 *bsrc = reinterpret_cast<const i32x4 *>(A.bias) + (eb >> 2);
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            if (s < n_used) {
                const i32x4 bv = bsrc[min(s * 64 + lane, nb - 1)];
                v[s].x = v[s].x == kI32Min ? kI32Min : sat_add_i32(v[s].x, bv.x);
                v[s].y = v[s].y == kI32Min ? kI32Min : sat_add_i32(v[s].y, bv.y);
                v[s].z = v[s].z == kI32Min ? kI32Min : sat_add_i32(v[s].z, bv.z);
                v[s].w = v[s].w == kI32Min ? kI32Min : sat_add_i32(v[s].w, bv.w);
            }
        }
    }

    // ---- elements outside the row become "minus infinity" (only a row's first block and the
    // passes that can reach its end need the test)
    int32_t x[SLOTS][4];
#pragma unroll
    for (int s = 0; s < SLOTS; ++s) {
        if (s >= n_used) {
            x[s][0] = x[s][1] = x[s][2] = x[s][3] = kI32Min;
            continue;
        }
        x[s][0] = v[s].x; x[s][1] = v[s].y; x[s][2] = v[s].z; x[s][3] = v[s].w;
        if (s == 0 || 4 * (s * 64 + 63) + 3 >= cols) {
            const int c0 = 4 * (s * 64 + lane) - phi;
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
    } else if (P.pre_mode == 2) {                     // shifts below 16: the general 64-bit form
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

    // ---- Eq. 6: row maximum
    int32_t mx = kI32Min;
#pragma unroll
    for (int s = 0; s < SLOTS; ++s) {
        if (s >= n_used) continue;
#pragma unroll
        for (int e = 0; e < 4; ++e) mx = max(mx, x[s][e]);
    }
    mx = group_max_i32<64>(mx);

    const int32_t D = P.d_clamp;
    const bool low_row = mx < kI32Min + D;            // wavefront-uniform here; see softmax_rows_kernel
    const int32_t lower = low_row ? kI32Min : mx - D;
    uint32_t w[SLOTS];                                // four output bytes per block
    if (P.variant == 0) softmax_slab_math<64, SLOTS, MODE, 0, POSTMODE, true>(x, w, mx, lower, low_row, lut, P, n_used);
    else softmax_slab_math<64, SLOTS, MODE, 1, POSTMODE, true>(x, w, mx, lower, low_row, lut, P, n_used);

    // ---- write back: whole blocks as dwords, the two shared edge blocks byte by byte
    uint8_t *dst8 = A.out + (e0 - phi);               // the byte of the row's first block, 4-byte aligned
#pragma unroll
    for (int s = 0; s < SLOTS; ++s) {
        if (s >= n_used) continue;
        const int b = s * 64 + lane;
        const int c0 = 4 * b - phi;
        if (s != 0 && 4 * (s * 64 + 63) + 3 < cols) {     // every lane's block lies inside the row
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

template <int SLOTS>
static void wide_launch_s(const WideArgs &A, int mode, int post_mode, dim3 grid, hipStream_t stream)
{
#define IPTQ_WIDE_LAUNCH(MODE, PM)                                                                \
    hipLaunchKernelGGL((softmax_wide_kernel<SLOTS, MODE, PM>), grid, dim3(256), 0, stream, A)
    if (mode == 0) {
        if (post_mode == PM_NONE) IPTQ_WIDE_LAUNCH(0, PM_NONE);
        else if (post_mode == PM_CLAMP127) IPTQ_WIDE_LAUNCH(0, PM_CLAMP127);
        else IPTQ_WIDE_LAUNCH(0, PM_GENERAL);
    } else {                                          // 2 covers 1: t16 == 0 shifts by 0
        if (post_mode == PM_NONE) IPTQ_WIDE_LAUNCH(2, PM_NONE);
        else if (post_mode == PM_CLAMP127) IPTQ_WIDE_LAUNCH(2, PM_CLAMP127);
        else IPTQ_WIDE_LAUNCH(2, PM_GENERAL);
    }
#undef IPTQ_WIDE_LAUNCH
}

// one translation unit per block count (softmax_wide_s<N>.hip)
void wide_launch_s8(const WideArgs &A, int mode, int post_mode, dim3 grid, hipStream_t stream);
void wide_launch_s13(const WideArgs &A, int mode, int post_mode, dim3 grid, hipStream_t stream);
void wide_launch_s16(const WideArgs &A, int mode, int post_mode, dim3 grid, hipStream_t stream);

}  // namespace iptq
