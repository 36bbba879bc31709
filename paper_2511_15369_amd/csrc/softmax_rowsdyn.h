// Integer softmax (Section 4.4, Eq. 6-15) for row lengths that have no compiled
// instantiation: the slab scheme and the register-resident arithmetic of the
// fixed-row-length kernel (softmax_rows.h) with the row length as a run-time value.  What is
// fixed at compile time is the lane layout: K lanes per row and exactly SLOTS 16-byte blocks
// per lane, SLOTS = ceil(B / K) with B the most blocks a row of that length can touch.  That
// pins down everything the code's shape depends on:
//   * a row touches B or B - 1 blocks, so the blocks of slots 0 .. SLOTS-2 exist in every
//     row and only the last slot's block index needs a clamp;
//   * a row's last (possibly cut) block lies in slot SLOTS-2 or SLOTS-1, its first in slot 0:
//     element masks and byte-wise output are confined to those three slots;
//   * the slab is SLOTS or SLOTS-1 passes of 64 chunks, of which all but the last two are
//     full: only those two clamp their chunk index.
// So the kernel has no branch that depends on the row length apart from lane predicates on
// LDS writes; the host instantiates one kernel per (K, SLOTS) and picks by row length.
#pragma once

#include <hip/hip_runtime.h>

#include <type_traits>

#include "device_common.h"
#include "kernels.h"
#include "plan.h"
#include "softmax_rows.h"

namespace iptq {

struct DynArgs {
    const int32_t *scores;
    const int32_t *bias;
    uint8_t *out;
    int64_t n_slabs;      // the last one may be partial
    int32_t tail_rows;    // rows of the last slab if it is partial, else 0
    int32_t cols;
    int32_t wave_lds;     // LDS bytes per wavefront: slab (16-byte multiple) + post table
    int32_t post_mode;    // PM_NONE / PM_CLAMP127 / PM_GENERAL, applied to the packed bytes
    // with an additive table: the wavefronts of a workgroup take slabs share_q apart, which read
    // the same table rows (see SoftmaxItem); 0: consecutive slabs
    uint32_t share_q, share_magic;
    int32_t share_sh;
    SoftmaxDev P;
};

template <int K, int SLOTS, int MODE>
__global__ void __launch_bounds__(256)
softmax_rowsdyn_kernel(DynArgs A)
{
    constexpr int RPW = 64 / K;                       // rows per wavefront, a multiple of 4
    extern __shared__ __attribute__((aligned(16))) uint8_t dyn_lds[];
    touch_kernel_arguments<sizeof(DynArgs)>();
    const SoftmaxDev &P = A.P;
    const int lane = threadIdx.x & 63;
    // (a scalar: the slab, its table offsets and every test on them then run on the scalar unit)
    const int wv = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const uint32_t wpb = blockDim.x >> 6;
    int64_t slab = (int64_t)blockIdx.x * wpb + wv;
    if (A.share_q != 0) {
        const uint32_t g = mulhi_u32(blockIdx.x, A.share_magic) >> A.share_sh;
        slab = (int64_t)g * (wpb * A.share_q) + (uint32_t)wv * A.share_q + (blockIdx.x - g * A.share_q);
    }
    if (slab >= A.n_slabs) return;                    // no workgroup barrier below

    const int cols = A.cols;
    const int slab_el = RPW * cols;                   // multiple of 4
    const int in_chunks = slab_el >> 2;               // in (64 (SLOTS-2), 64 SLOTS]
    uint8_t *lds = dyn_lds + wv * A.wave_lds;
    uint8_t *lut = lds + A.wave_lds - kPostLutBytes;
    const int post_mode = A.post_mode;
    if (post_mode == PM_GENERAL) {                    // ordered before its use by the fences below
        const int p_max = 1 << (P.m_bits - P.p_shift);
        for (int p = lane; p <= p_max; p += 64) lut[p] = (uint8_t)post_dev<PM_GENERAL>((uint32_t)p, P);
    }
    const int32_t *src1 = A.scores + slab * slab_el;
    const int32_t *__restrict__ bias = A.bias;
    const bool partial = A.tail_rows != 0 && slab == A.n_slabs - 1;
    const int valid_el = (partial ? A.tail_rows : RPW) * cols;

    // ---- flat copy of the slab into LDS, bias added on the way.  Every load is issued before
    // the first LDS write and none sits behind a branch: in the last two passes the lanes
    // beyond the slab's last chunk load that chunk again and write it to its place again.
    auto add_bias = [](i32x4 v, const i32x4 bv) {
        v = add_table_chunk(v, bv);
        return v;
    };
    // With a table the scores are added with the saturating sum alone, which is the exact value
    // unless a score or an entry is INT32_MIN, and the smallest operand is tracked beside it (two
    // lane-ops per score instead of four); returns whether any lane met INT32_MIN, in which case
    // the caller copies the slab in again with the exact rule.
    auto copy_in = [&](auto bias_tag, auto straddle_tag) -> bool {
        constexpr bool BIAS = decltype(bias_tag)::value;
        i32x4 lowest = {0, 0, 0, 0};
        // the additive table's size is not a multiple of four scores and its end falls inside
        // this slab: one chunk takes entries from both ends of the table
        constexpr bool STRADDLE = decltype(straddle_tag)::value;
        i32x4 *lds4 = reinterpret_cast<i32x4 *>(lds);
        const int last = in_chunks - 1;
        auto chunk_of = [&](int i) {
            const int idx = i * 64 + lane;
            return i >= SLOTS - 2 ? min(idx, last) : idx;
        };
        uint32_t boff = 0;
        if (BIAS) boff = row_mod_period((uint32_t)(slab * RPW), P) * (uint32_t)cols;
        const uint32_t pe = (uint32_t)P.bias_period_rows * (uint32_t)cols;
        // bias chunks come from L2: a ring of kAhead loads in flight behind the score loads
        // keeps the staging registers at 4 * (SLOTS + kAhead)
        constexpr int kAhead = 4;
        i32x4 first4 = {0, 0, 0, 0};
        if (STRADDLE) first4 = load_i32x4(bias);
        auto bias_chunk = [&](int i) {
            uint32_t o = boff + 4u * (uint32_t)chunk_of(i);
            if (o >= pe) o -= pe;
            return STRADDLE ? bias_chunk_wrapping(bias, o, pe, first4) : load_i32x4(bias + o);
        };
        i32x4 v[SLOTS], bv[BIAS ? kAhead : 1];
#pragma unroll
        for (int i = 0; i < SLOTS; ++i) v[i] = stream_load_i32x4(src1 + 4 * chunk_of(i));
        if (BIAS) {
#pragma unroll
            for (int i = 0; i < kAhead && i < SLOTS; ++i) bv[i] = bias_chunk(i);
        }
#pragma unroll
        for (int i = 0; i < SLOTS; ++i) {
            i32x4 t = v[i];
            if (BIAS) {
                const i32x4 b = bv[i % kAhead];
                lowest.x = min(min(lowest.x, t.x), b.x);
                lowest.y = min(min(lowest.y, t.y), b.y);
                lowest.z = min(min(lowest.z, t.z), b.z);
                lowest.w = min(min(lowest.w, t.w), b.w);
                t.x = sat_add_i32(t.x, b.x);
                t.y = sat_add_i32(t.y, b.y);
                t.z = sat_add_i32(t.z, b.z);
                t.w = sat_add_i32(t.w, b.w);
            }
            if (BIAS && i + kAhead < SLOTS) bv[i % kAhead] = bias_chunk(i + kAhead);
            lds4[chunk_of(i)] = t;
        }
        wave_lds_fence();
        return BIAS && __builtin_amdgcn_ballot_w64(min(min(lowest.x, lowest.y), min(lowest.z, lowest.w)) == kI32Min) != 0;
    };
    // the one partial slab of a launch, and a slab that holds an INT32_MIN operand: guarded loads
    // and the exact addition, chunk by chunk
    auto copy_in_partial = [&]() {
        i32x4 *lds4 = reinterpret_cast<i32x4 *>(lds);
        uint32_t boff = 0;
        if (bias != nullptr) boff = row_mod_period((uint32_t)(slab * RPW), P) * (uint32_t)cols;
        const uint32_t pe = (uint32_t)P.bias_period_rows * (uint32_t)cols;
        for (int idx = lane; idx < in_chunks; idx += 64) {
            i32x4 v;
            if (4 * idx + 3 < valid_el) {
                v = stream_load_i32x4(src1 + 4 * idx);
            } else {
                v = (i32x4){0, 0, 0, 0};
                if (4 * idx < valid_el) v.x = src1[4 * idx];
                if (4 * idx + 1 < valid_el) v.y = src1[4 * idx + 1];
                if (4 * idx + 2 < valid_el) v.z = src1[4 * idx + 2];
            }
            if (bias != nullptr) {
                uint32_t o = boff + 4u * (uint32_t)idx;
                if (o >= pe) o -= pe;
                v = add_bias(v, bias_chunk_wrapping(bias, o, pe, load_i32x4(bias)));
            }
            lds4[idx] = v;
        }
        wave_lds_fence();
    };
    if (__builtin_expect(partial, 0)) copy_in_partial();
    else if (bias == nullptr) copy_in(std::false_type{}, std::false_type{});
    else {
        const uint32_t pe = (uint32_t)P.bias_period_rows * (uint32_t)cols;
        const uint32_t boff = row_mod_period((uint32_t)(slab * RPW), P) * (uint32_t)cols;
        bool redo;
        if ((pe & 3u) != 0 && boff + (uint32_t)slab_el > pe) redo = copy_in(std::true_type{}, std::true_type{});
        else redo = copy_in(std::true_type{}, std::false_type{});
        if (__builtin_expect(redo, 0)) copy_in_partial();
    }

    // ---- this lane's blocks; elements outside the row become "minus infinity"
    const int lr = lane / K;                          // row inside the slab
    const int j = lane % K;                           // lane inside the row
    const int e_r = lr * cols;                        // first element of the row in the slab
    const int b_r = e_r >> 2;                         // its 16-byte block
    const int phi = e_r & 3;                          // and its offset inside that block
    const int nb = (phi + cols + 3) >> 2;             // blocks the row touches
    auto edge_slot = [](int s) { return s == 0 || s >= SLOTS - 2; };
    int32_t x[SLOTS][4];
#pragma unroll
    for (int s = 0; s < SLOTS; ++s) {
        const int b = s * K + j;
        // a block beyond the row's last one (last slot only) is read from the last one and
        // masked entirely below: no lane-divergent branch around the LDS read
        const int bb = s == SLOTS - 1 ? min(b, nb - 1) : b;
        const i32x4 v = reinterpret_cast<const i32x4 *>(lds)[b_r + bb];
        x[s][0] = v.x; x[s][1] = v.y; x[s][2] = v.z; x[s][3] = v.w;
        if (edge_slot(s)) {
            const int c0 = 4 * b - phi;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if ((unsigned)(c0 + e) >= (unsigned)cols) x[s][e] = kI32Min;
        }
    }
    wave_lds_fence();                                 // the slab area is reused for the output

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
    mx = group_max_i32<K>(mx);

    const int32_t D = P.d_clamp;
    const bool low_row = mx < kI32Min + D;            // see softmax_rows_kernel
    const int32_t lower = low_row ? kI32Min : mx - D;
    const bool any_low = __builtin_amdgcn_ballot_w64(low_row) != 0;
    uint32_t w[SLOTS];                                // four probabilities per block, one per byte

    if (P.variant == 0) softmax_slab_math<K, SLOTS, MODE, 0, PM_NONE>(x, w, mx, lower, any_low, lut, P);
    else softmax_slab_math<K, SLOTS, MODE, 1, PM_NONE>(x, w, mx, lower, any_low, lut, P);

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

    // ---- assemble the slab's bytes in LDS
    uint32_t *lds32 = reinterpret_cast<uint32_t *>(lds);
#pragma unroll
    for (int s = 0; s < SLOTS; ++s) {
        const int b = s * K + j;
        if (!edge_slot(s)) {                          // every lane's block lies inside its row
            lds32[b_r + b] = w[s];
        } else if (b < nb) {
            const int c0 = 4 * b - phi;
            if (c0 >= 0 && c0 + 3 < cols) {
                lds32[b_r + b] = w[s];
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if ((unsigned)(c0 + e) < (unsigned)cols)
                        lds[4 * (b_r + b) + e] = (uint8_t)(w[s] >> (8 * e));
            }
        }
    }
    wave_lds_fence();

    // ---- flat, fully coalesced store (byte stores at the end of a partial slab)
    uint8_t *dst8 = A.out + slab * slab_el;
    if ((slab_el & 15) == 0) {
        const int n16 = slab_el >> 4;
#pragma unroll
        for (int i = 0; i < (SLOTS + 3) / 4; ++i) {
            const int idx = i * 64 + lane;
            if (idx < n16) {
                if (16 * idx + 15 < valid_el) {
                    stream_store_bytes16(reinterpret_cast<const u32x4 *>(lds)[idx], dst8 + 16 * idx);
                } else {
#pragma unroll 1
                    for (int b = 16 * idx; b < valid_el && b < 16 * idx + 16; ++b) dst8[b] = lds[b];
                }
            }
        }
    } else {
#pragma unroll
        for (int i = 0; i < SLOTS; ++i) {
            const int idx = i * 64 + lane;
            if (idx < in_chunks) {
                if (4 * idx + 3 < valid_el) {
                    stream_store_bytes4(lds32[idx], dst8 + 4 * idx);
                } else {
#pragma unroll 1
                    for (int b = 4 * idx; b < valid_el && b < 4 * idx + 4; ++b) dst8[b] = lds[b];
                }
            }
        }
    }
}

// mode: SoftmaxDev::mode16 (2 covers 1: t16 == 0 shifts by 0)
template <int K, int SLOTS>
static void rowsdyn_launch_ks(const DynArgs &A, int mode, dim3 grid, dim3 block, size_t lds, hipStream_t stream)
{
    if (mode == 0) hipLaunchKernelGGL((softmax_rowsdyn_kernel<K, SLOTS, 0>), grid, block, lds, stream, A);
    else hipLaunchKernelGGL((softmax_rowsdyn_kernel<K, SLOTS, 2>), grid, block, lds, stream, A);
}

// One launcher per group of layouts, each defined in its own translation unit so that the
// instantiations compile in parallel.  Each returns false for a slot count it does not hold.
bool rowsdyn_launch_k1(const DynArgs &, int slots, int mode, dim3, dim3, size_t, hipStream_t);         // 1..8
bool rowsdyn_launch_k2(const DynArgs &, int slots, int mode, dim3, dim3, size_t, hipStream_t);         // 5..8
bool rowsdyn_launch_k4(const DynArgs &, int slots, int mode, dim3, dim3, size_t, hipStream_t);         // 5..8
bool rowsdyn_launch_k8(const DynArgs &, int slots, int mode, dim3, dim3, size_t, hipStream_t);         // 5..8
bool rowsdyn_launch_k16(const DynArgs &, int slots, int mode, dim3, dim3, size_t, hipStream_t);        // 5..8
bool rowsdyn_launch_k16_long(const DynArgs &, int slots, int mode, dim3, dim3, size_t, hipStream_t);   // 9..10

#define IPTQ_ROWSDYN_CASE(K, S)                                                                   \
    case S: rowsdyn_launch_ks<K, S>(A, mode, grid, block, lds, stream); return true;

}  // namespace iptq
