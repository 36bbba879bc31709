// Integer softmax kernels for gfx950 (Section 4.4, Eq. 6-15).
//
// Two kernel families compute the same function:
//   softmax_rows_kernel  - compile-time row length, a fixed number K of lanes per row so
//                          that a wavefront owns 64/K whole rows (a "slab").  The slab is
//                          contiguous and 16-byte aligned in both the int32 input and the
//                          byte output, so every global access is a full dwordx4.  Rows
//                          are addressed on the 16-byte grid of the flat tensor ("blocks"
//                          of 4 elements); a row that does not start on that grid simply
//                          ignores the neighbours' elements in its first and last block.
//   softmax_generic_kernel - run-time row length, one wavefront per row, three passes.
//                          Serves odd shapes, the tail rows of the first family and the
//                          fused pre-requantization.
#include <hip/hip_runtime.h>

#include "device_common.h"
#include "plan.h"

namespace iptq {

// One exponential (Eq. 7-10 / 13-14).  x is the (biased, requantized) score, `lower` is
// max(row) - D saturated, mx the row maximum.  Elements at or below `lower` get the same
// all-zero result as their true value, which keeps every intermediate inside 32 bits.
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
    if (VARIANT == 1) fr += (nr >> 3) + (nr >> 4);     // Eq. 13: (0.1011)b x
    const uint32_t base = ((uint32_t)fr << P.n_shift) + (uint32_t)P.i0n;  // Eq. 14, << N
    uint32_t e = base >> q;                            // Eq. 9 (q <= 31 by the clamp)
    if (EXPLICIT_MASK) e = (x == kI32Min) ? 0u : e;
    return e;
}

template <int POSTMODE>
IPTQ_DEV uint32_t post_dev(uint32_t p, const SoftmaxDev &P)
{
    if (POSTMODE == 0) return p;                                   // identity, cannot clip
    if (POSTMODE == 1) return min(p, (uint32_t)P.qmax);            // identity, clip at qmax
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

// ---------------------------------------------------------------------------------------
// Fixed row length.  COLS: row length; K: lanes per row; STAGE: copy the slab through LDS
// with flat coalesced loads (needed when K is small, otherwise lanes read their blocks
// straight from global memory); BIAS: additive bias (STAGE only); POSTMODE as above.
template <int COLS, int K, bool STAGE, int VARIANT, bool BIAS, int POSTMODE>
__global__ void __launch_bounds__(256)
softmax_rows_kernel(const int32_t *__restrict__ scores, const int32_t *__restrict__ bias,
                    uint8_t *__restrict__ out, int64_t n_slabs, SoftmaxDev P)
{
    constexpr int RPW = 64 / K;                       // rows per wavefront
    constexpr int SLAB = RPW * COLS;                  // elements per slab
    static_assert(SLAB % 16 == 0, "slab must be 16-byte aligned in the byte output");
    static_assert(!BIAS || STAGE, "bias is fused into the staging copy");
    constexpr int NB = (COLS + 3 + 3) / 4;            // 16-byte blocks a row can touch
    constexpr int SLOTS = (NB + K - 1) / K;           // blocks per lane
    constexpr int IN_CHUNKS = SLAB / 4;               // 16-byte chunks of the input slab
    constexpr int OUT_CHUNKS = SLAB / 16;             // 16-byte chunks of the output slab
    constexpr int LDS_BYTES = STAGE ? SLAB * 4 : SLAB;
    __shared__ __attribute__((aligned(16))) uint8_t lds_all[4][LDS_BYTES];

    const int lane = threadIdx.x & 63;
    const int wv = threadIdx.x >> 6;
    const int64_t slab = (int64_t)blockIdx.x * 4 + wv;
    if (slab >= n_slabs) return;                      // no workgroup barrier below

    uint8_t *lds = lds_all[wv];
    const i32x4 *src = reinterpret_cast<const i32x4 *>(scores + slab * SLAB);
    const int lr = lane / K;                          // row inside the slab
    const int j = lane % K;                           // lane inside the row
    const int e_r = lr * COLS;                        // first element of the row in the slab
    const int b_r = e_r >> 2;                         // its 16-byte block
    const int phi = e_r & 3;                          // and its offset inside that block

    if (STAGE) {
        i32x4 *lds4 = reinterpret_cast<i32x4 *>(lds);
        uint32_t boff = 0;
        if (BIAS) boff = row_mod_period((uint32_t)(slab * RPW), P) * (uint32_t)COLS;
        const uint32_t pe = (uint32_t)P.bias_period_rows * (uint32_t)COLS;
#pragma unroll
        for (int i = 0; i < (IN_CHUNKS + 63) / 64; ++i) {
            const int idx = i * 64 + lane;
            if ((i + 1) * 64 <= IN_CHUNKS || idx < IN_CHUNKS) {
                i32x4 v = stream_load(src + idx);
                if (BIAS) {
                    uint32_t o = boff + 4u * (uint32_t)idx;
                    if (o >= pe) o -= pe;
                    const i32x4 bv = *reinterpret_cast<const i32x4 *>(bias + o);
                    v.x = v.x == kI32Min ? v.x : sat_add_i32(v.x, bv.x);
                    v.y = v.y == kI32Min ? v.y : sat_add_i32(v.y, bv.y);
                    v.z = v.z == kI32Min ? v.z : sat_add_i32(v.z, bv.z);
                    v.w = v.w == kI32Min ? v.w : sat_add_i32(v.w, bv.w);
                }
                lds4[idx] = v;
            }
        }
        wave_lds_fence();
    }

    // ---- load this lane's blocks; elements outside the row become "minus infinity"
    int32_t x[SLOTS][4];
#pragma unroll
    for (int s = 0; s < SLOTS; ++s) {
        const int b = s * K + j;
        const bool always_inside = 4 * (s * K + K - 1) < COLS;    // block overlaps the row for every lane
        i32x4 v = {kI32Min, kI32Min, kI32Min, kI32Min};
        if (always_inside || 4 * b < phi + COLS) {
            if (STAGE) v = reinterpret_cast<const i32x4 *>(lds)[b_r + b];
            else v = stream_load(src + b_r + b);
        }
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
    if (STAGE) wave_lds_fence();                      // the slab area is reused for the output

    // ---- Eq. 6: row maximum
    int32_t mx = kI32Min;
#pragma unroll
    for (int s = 0; s < SLOTS; ++s)
#pragma unroll
        for (int e = 0; e < 4; ++e) mx = max(mx, x[s][e]);
    mx = group_max_i32<K>(mx);

    // Rows whose maximum lies within D of INT32_MIN cannot use the clamp to zero out
    // masked entries; the whole wavefront then takes the path with an explicit test.
    const int32_t D = P.d_clamp;
    const bool low_row = mx < kI32Min + D;
    const int32_t lower = low_row ? kI32Min : mx - D;
    uint32_t sum = 0;
    if (__builtin_amdgcn_ballot_w64(low_row) == 0) {
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
    sum = group_sum_u32<K>(sum);

    // ---- Eq. 15: one reciprocal per row, then multiply and shift
    const uint32_t f = floor_pow2_div(P.m_bits, sum);
    uint32_t *lds32 = reinterpret_cast<uint32_t *>(lds);
#pragma unroll
    for (int s = 0; s < SLOTS; ++s) {
        const int b = s * K + j;
        uint32_t pk = 0;
        uint32_t pb[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t p = ((uint32_t)x[s][e] * f) >> P.p_shift;
            pb[e] = post_dev<POSTMODE>(p, P);
            pk |= pb[e] << (8 * e);
        }
        const bool always_full = (s != 0) && (4 * (s * K + K - 1) + 3 < COLS);
        if (always_full) {
            lds32[b_r + b] = pk;
        } else {
            const int c0 = 4 * b - phi;
            if (c0 >= 0 && c0 + 3 < COLS) {
                lds32[b_r + b] = pk;
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if ((unsigned)(c0 + e) < (unsigned)COLS) lds[4 * (b_r + b) + e] = (uint8_t)pb[e];
            }
        }
    }
    wave_lds_fence();

    // ---- flat, fully coalesced store of the slab's bytes
    u32x4 *dst = reinterpret_cast<u32x4 *>(out + slab * SLAB);
    const u32x4 *lds4o = reinterpret_cast<const u32x4 *>(lds);
#pragma unroll
    for (int i = 0; i < (OUT_CHUNKS + 63) / 64; ++i) {
        const int idx = i * 64 + lane;
        if ((i + 1) * 64 <= OUT_CHUNKS || idx < OUT_CHUNKS)
            stream_store(lds4o[idx], dst + idx);
    }
}

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
        orow[c] = (uint8_t)post_dev<2>(p, P);
    }
}

// ---------------------------------------------------------------------------------------
// Host-side dispatch.

static int post_mode_of(const SoftmaxDev &P, int out_bits)
{
    const bool identity = P.post_m == 1 && P.post_s == 0 && P.post_zp == 0 && P.qmin <= 0;
    if (!identity) return 2;
    return P.qmax >= (1 << (out_bits - 1)) ? 0 : 1;
}

template <int COLS, int K, bool STAGE, int VARIANT, bool BIAS>
static hipError_t launch_rows_post(int post_mode, const int32_t *scores, const int32_t *bias,
                                   uint8_t *out, int64_t n_slabs, const SoftmaxDev &P,
                                   hipStream_t stream)
{
    const dim3 grid((unsigned)((n_slabs + 3) / 4)), block(256);
    switch (post_mode) {
    case 0:
        hipLaunchKernelGGL((softmax_rows_kernel<COLS, K, STAGE, VARIANT, BIAS, 0>), grid, block, 0,
                           stream, scores, bias, out, n_slabs, P);
        break;
    case 1:
        hipLaunchKernelGGL((softmax_rows_kernel<COLS, K, STAGE, VARIANT, BIAS, 1>), grid, block, 0,
                           stream, scores, bias, out, n_slabs, P);
        break;
    default:
        hipLaunchKernelGGL((softmax_rows_kernel<COLS, K, STAGE, VARIANT, BIAS, 2>), grid, block, 0,
                           stream, scores, bias, out, n_slabs, P);
        break;
    }
    return hipGetLastError();
}

template <int COLS, int K, bool STAGE>
static hipError_t launch_rows(int post_mode, bool has_bias, const int32_t *scores,
                              const int32_t *bias, uint8_t *out, int64_t n_slabs,
                              const SoftmaxDev &P, hipStream_t stream)
{
    if constexpr (STAGE) {
        if (has_bias) {
            return P.variant == 0
                       ? launch_rows_post<COLS, K, STAGE, 0, true>(post_mode, scores, bias, out, n_slabs, P, stream)
                       : launch_rows_post<COLS, K, STAGE, 1, true>(post_mode, scores, bias, out, n_slabs, P, stream);
        }
    }
    return P.variant == 0
               ? launch_rows_post<COLS, K, STAGE, 0, false>(post_mode, scores, bias, out, n_slabs, P, stream)
               : launch_rows_post<COLS, K, STAGE, 1, false>(post_mode, scores, bias, out, n_slabs, P, stream);
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
        if (cols == 197 && !has_bias) {
            const int64_t n_slabs = rows / 16;
            if (n_slabs > 0) err = launch_rows<197, 4, false>(post_mode, false, scores, bias, out, n_slabs, P, stream);
            done = n_slabs * 16;
        } else if (cols == 197 && bias_ok(16)) {
            const int64_t n_slabs = rows / 16;
            if (n_slabs > 0) err = launch_rows<197, 4, true>(post_mode, true, scores, bias, out, n_slabs, P, stream);
            done = n_slabs * 16;
        } else if (cols == 49 && bias_ok(64)) {
            const int64_t n_slabs = rows / 64;
            if (n_slabs > 0) err = launch_rows<49, 1, true>(post_mode, has_bias, scores, bias, out, n_slabs, P, stream);
            done = n_slabs * 64;
        }
        if (err != hipSuccess) return err;
    }
    return launch_generic(scores, bias, out, done, rows, cols, has_bias, has_pre, P, stream);
}

}  // namespace iptq
