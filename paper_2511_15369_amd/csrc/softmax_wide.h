// Integer softmax (Section 4.4, Eq. 6-15) for long rows: one wavefront per row, the row
// held in registers, no LDS staging.  All 64 lanes share the row: lane l of pass s owns the
// 16-byte block s * 64 + l of the aligned block range that covers the row, so a pass is one
// fully coalesced 1 KiB load.  A row that does not start on a 16-byte boundary shares its first
// and last block with its neighbours: their elements are masked on the way in and those
// blocks are written back with byte stores, every other block with one dword store at whatever
// byte address it has (so the tensor may start anywhere on the 4-byte grid and the output
// anywhere at all).  The
// arithmetic is the slab kernels' (softmax_slab_math with 64 lanes per row).
// SLOTS is exactly the number of passes a row of this length needs at its worst alignment,
// ceil(B / 64) with B the most blocks it can touch: a row touches B or B - 1 blocks, so the
// blocks of passes 0 .. SLOTS-2 exist in every row, only the last pass clamps its block
// index (the last two do: one instruction), and only passes 0, SLOTS-2 and SLOTS-1 can hold a
// row's first or last block (element masks, byte stores).  No branch depends on the row
// length.
#pragma once

#include <hip/hip_runtime.h>

#include "device_common.h"
#include "kernels.h"
#include "plan.h"
#include "softmax_rows.h"

namespace iptq {

struct WideArgs {
    const int32_t *scores;   // the tensor's address rounded down to 16 bytes
    const int32_t *bias;     // NULL or 16-byte aligned, period * cols a multiple of 4 (base_off == 0 then)
    uint8_t *out;            // the output's address minus base_off (any byte address)
    int64_t rows;
    int32_t base_off;        // scores between the rounded-down address and the tensor: 0..3
    int32_t cols;            // >= 8 when cut_el != 0 (host)
    int32_t cut_el;          // scores in the tensor's final 16-byte block if the tensor ends off the
                             // 16-byte grid (the last row must not load that block whole), else 0
    int32_t post_mode;       // PM_NONE / PM_CLAMP127 / PM_GENERAL, applied to the packed bytes
    SoftmaxDev P;
};

template <int SLOTS, int MODE>
__global__ void __launch_bounds__(256)
softmax_wide_kernel(WideArgs A)
{
    __shared__ uint8_t lut_all[4][kPostLutBytes];
    touch_kernel_arguments<sizeof(WideArgs)>();
    const SoftmaxDev P = A.P;
    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));   // the row index as a scalar
    const int64_t row = (int64_t)blockIdx.x * 4 + wv;
    if (row >= A.rows) return;                        // no workgroup barrier below

    uint8_t *lut = lut_all[wv];
    const int post_mode = A.post_mode;
    if (post_mode == PM_GENERAL) {
        const int p_max = 1 << (P.m_bits - P.p_shift);
        for (int p = lane; p <= p_max; p += 64) lut[p] = (uint8_t)post_dev<PM_GENERAL>((uint32_t)p, P);
        wave_lds_fence();
    }

    const int cols = A.cols;
    const int64_t e0 = row * cols + A.base_off;       // the row's first element on the 16-byte grid
    const int phi = (int)(e0 & 3);                    // its offset inside its 16-byte block
    const int nb = (phi + cols + 3) >> 2;             // blocks the row touches (wavefront-uniform)
    const i32x4 *src = reinterpret_cast<const i32x4 *>(A.scores) + (e0 >> 2);
    // the last row of a tensor that ends off the 16-byte grid: its final block is loaded
    // element by element below (wavefront-uniform case)
    const bool cut = A.cut_el != 0 && row == A.rows - 1;
    const int nb_whole = cut ? nb - 1 : nb;           // blocks that can be loaded whole, >= 1
    auto block_of = [&](int s, int n) {               // lanes beyond block n - 1 load it again
        const int b = s * 64 + lane;
        return s >= SLOTS - 2 ? min(b, n - 1) : b;
    };
    auto edge_slot = [](int s) { return s == 0 || s >= SLOTS - 2; };

    // ---- the row's blocks; every load is issued before the first use and none sits behind a
    // branch
    i32x4 v[SLOTS];
#pragma unroll
    for (int s = 0; s < SLOTS; ++s) v[s] = stream_load(src + block_of(s, nb_whole));
    if (cut) {
        const int32_t *last = reinterpret_cast<const int32_t *>(src + (nb - 1));
#pragma unroll
        for (int s = SLOTS >= 2 ? SLOTS - 2 : 0; s < SLOTS; ++s) {
            if (s * 64 + lane == nb - 1) {            // elements beyond cut_el are masked below
                v[s].x = last[0];
                if (A.cut_el > 1) v[s].y = last[1];
                if (A.cut_el > 2) v[s].z = last[2];
            }
        }
    }
    if (A.bias != nullptr) {
        // the bias row starts at the same offset inside a block (period * cols % 4 == 0)
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
    mx = group_max_i32<64>(mx);

    const int32_t D = P.d_clamp;
    const bool low_row = mx < kI32Min + D;            // wavefront-uniform here; see softmax_rows_kernel
    const int32_t lower = low_row ? kI32Min : mx - D;
    uint32_t w[SLOTS];                                // four probabilities per block, one per byte
    if (P.variant == 0) softmax_slab_math<64, SLOTS, MODE, 0, PM_NONE>(x, w, mx, lower, low_row, lut, P);
    else softmax_slab_math<64, SLOTS, MODE, 1, PM_NONE>(x, w, mx, lower, low_row, lut, P);

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
    uint8_t *dst8 = A.out + (e0 - phi);               // the byte of the row's first block
#pragma unroll
    for (int s = 0; s < SLOTS; ++s) {
        const int b = s * 64 + lane;
        const int c0 = 4 * b - phi;
        if (!edge_slot(s)) {                          // every lane's block lies inside the row
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
template <int SLOTS>
static void wide_launch_s(const WideArgs &A, int mode, dim3 grid, hipStream_t stream)
{
    if (mode == 0) hipLaunchKernelGGL((softmax_wide_kernel<SLOTS, 0>), grid, dim3(256), 0, stream, A);
    else hipLaunchKernelGGL((softmax_wide_kernel<SLOTS, 2>), grid, dim3(256), 0, stream, A);
}

// one translation unit per group of pass counts; each returns false for a count it does not hold
bool wide_launch_p1_6(const WideArgs &A, int passes, int mode, dim3 grid, hipStream_t stream);
bool wide_launch_p7_10(const WideArgs &A, int passes, int mode, dim3 grid, hipStream_t stream);
bool wide_launch_p11_13(const WideArgs &A, int passes, int mode, dim3 grid, hipStream_t stream);
bool wide_launch_p14_16(const WideArgs &A, int passes, int mode, dim3 grid, hipStream_t stream);

#define IPTQ_WIDE_CASE(S)                                                                         \
    case S: wide_launch_s<S>(A, mode, grid, stream); return true;

}  // namespace iptq
