// Element-wise integer kernels for gfx950: polynomial GELU (Section 4.3, Eq. 3 and 5) and
// the dyadic requantization.  All of them stream: each 16-byte chunk is read once and
// written once with dwordx4 accesses.
#include <hip/hip_runtime.h>

#include "device_common.h"
#include "kernels.h"
#include "plan.h"

namespace iptq {

// One GELU value.  `in` is the already requantized input code.
//   q = clamp(in - zp, +-max_abs_q); t = min(|q|, -q_b) + q_b; t^p (square reused);
//   v = (sign(q) (t^p + q_c) + q_c) >> k; w = q v; y = requant(w).
// For q >= 0 the numerator is t^p + 2 q_c; for q < 0 it is -t^p, and
// floor(-a / 2^k) == ~floor((a - 1) / 2^k), so both signs share one 64-bit add and shift.
template <bool NARROW>
IPTQ_DEV int32_t gelu_eval_dev(int32_t in, const GeluDev &P)
{
    int32_t q = in - P.zp_in;                       // |in|, |zp| small enough on both entries
    q = min(max(q, -P.max_abs_q), P.max_abs_q);
    const int32_t aq = max(q, -q);
    const int32_t t = min(aq, -P.q_b) + P.q_b;      // Eq. 3: clip at -b, add b
    const int64_t t2 = (int64_t)t * (int64_t)t;     // < 2^30 for the quartic, < 2^60 otherwise
    const int64_t tp = P.quartic ? (int64_t)((uint64_t)(uint32_t)t2 * (uint64_t)(uint32_t)t2) : t2;
    const bool neg = q < 0;
    const int64_t addend = neg ? (int64_t)-1 : 2 * P.q_c;
    const int64_t z = (tp + addend) >> P.k;
    const int32_t v = neg ? ~(int32_t)z : (int32_t)z;
    const int32_t w = q * v;                        // Eq. 5: x (1 + L); 1/2 is in the scale
    return requant_dev<NARROW>(w, P.post_m, P.post_s, P.post_zp, P.qmin, P.qmax);
}

// The same value by a shorter route, for the usual case GeluDev::fast (t^2 < 2^31 and
// post_s >= 16).  q is the centred, clamped input.  The sign of q turns into a mask: the
// addend (2 q_c or -1) is an OR with it, the final negation an XOR, and t^4 + addend is one
// 64-bit multiply-add.
template <bool QUARTIC>
IPTQ_DEV int32_t gelu_eval_fast(int32_t q, const GeluDev &P)
{
    const int32_t aq = max(q, -q);
    const int32_t t = min(aq, -P.q_b) + P.q_b;               // Eq. 3: clip at -b, add b
    const uint32_t t2 = (uint32_t)(t * t);
    const uint32_t mask = (uint32_t)(q >> 31);               // all ones for q < 0
    const uint64_t qc2 = (uint64_t)(2 * P.q_c);
    const uint64_t addend = ((uint64_t)((uint32_t)(qc2 >> 32) | mask) << 32) | ((uint32_t)qc2 | mask);
    const uint64_t tp = QUARTIC ? (uint64_t)t2 * (uint64_t)t2 + addend : (uint64_t)t2 + addend;
    const int32_t v = (int32_t)((int64_t)tp >> P.k) ^ (int32_t)mask;
    const int32_t w = q * v;                                 // Eq. 5
    const int64_t r = (int64_t)w * (int64_t)P.post_m + ((int64_t)1 << (P.post_s - 1));
    const int32_t y = (int32_t)(r >> P.post_s) + P.post_zp;
    return clamp_i32(y, P.qmin, P.qmax);
}

IPTQ_DEV int32_t gelu_eval_any(int32_t in, const GeluDev &P)
{
    return P.post_s >= 16 ? gelu_eval_dev<true>(in, P) : gelu_eval_dev<false>(in, P);
}

IPTQ_DEV uint32_t pack4(int32_t a, int32_t b, int32_t c, int32_t d)
{
    return ((uint32_t)a & 0xffu) | (((uint32_t)b & 0xffu) << 8) | (((uint32_t)c & 0xffu) << 16) |
           ((uint32_t)d << 24);
}

IPTQ_DEV int32_t sbyte(uint32_t w, int i) { return (int32_t)(int8_t)(w >> (8 * i)); }

// ---------------------------------------------------------------------------------------
// int8 -> int8 through a per-workgroup table: the polynomial is evaluated once for each of
// the 256 input codes with the exact integer formula, then every element is one byte
// gather from LDS.  One launch serves up to kGeluBatchMax independent problems (the layers
// of a sweep): workgroups [first_wg, first_wg + n_wgs) stream item i.  The last (n & 15)
// bytes of an item are done by its first workgroup.  `out` is 16-byte aligned: the host
// peels the `head` bytes in front of that boundary off the tensor (the item's first
// workgroup does them too).  `in` is then aligned as well if the two tensors sit at the same
// offset (in place, or views cut at the same element); if not, its 16-byte loads are
// unaligned ones.  in and out may be the same buffer.
constexpr int kGeluBatchMax = 16;
constexpr int64_t kGeluTableGridCap = 256 * 56;
struct GeluItem {
    const uint8_t *in;
    uint8_t *out;
    int64_t n;
    uint32_t first_wg;
    uint32_t n_wgs;
    uint32_t head;          // bytes in front of in / out that belong to the tensor: 0..15
    GeluDev P;
};
struct GeluBatch {
    int32_t n_items;
    GeluItem item[kGeluBatchMax];
};
static_assert(sizeof(GeluBatch) <= 4096, "kernel arguments are limited to 4 KiB");

__global__ void __launch_bounds__(256)
gelu_i8_table_kernel(GeluBatch B)
{
    touch_kernel_arguments<8 + sizeof(GeluItem)>();       // the batch header and its first problem
    int it = 0;
    for (int i = 1; i < B.n_items; ++i)
        if (blockIdx.x >= B.item[i].first_wg) it = i;
    const GeluItem &I = B.item[it];
    __shared__ uint8_t table[256];
    const int64_t n = I.n;
    const int64_t n16 = n >> 4;
    u32x4 *out4 = reinterpret_cast<u32x4 *>(I.out);
    const uint32_t lb = blockIdx.x - I.first_wg;
    const int64_t stride = (int64_t)I.n_wgs * 256;
    auto gather = [&](const u32x4 v) -> u32x4 {
        u32x4 r;
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const uint32_t w = v[d];
            const uint32_t y0 = table[w & 0xffu];
            const uint32_t y1 = table[(w >> 8) & 0xffu];
            const uint32_t y2 = table[(w >> 16) & 0xffu];
            const uint32_t y3 = table[w >> 24];
            r[d] = y0 | (y1 << 8) | (y2 << 16) | (y3 << 24);
        }
        return r;
    };
    // the same global_load_dwordx4 serves an input on the 16-byte grid and one off it
    typedef u32x4 __attribute__((aligned(1))) u32x4_unaligned;
    const u32x4_unaligned *in4u = reinterpret_cast<const u32x4_unaligned *>(I.in);
    auto load16 = [&](int64_t k) -> u32x4 { return __builtin_nontemporal_load(in4u + k); };
    int64_t i = (int64_t)lb * 256 + threadIdx.x;
    // the first chunk's load is in flight while the table is built
    u32x4 first = {0u, 0u, 0u, 0u};
    if (i < n16) first = load16(i);
    table[threadIdx.x] = (uint8_t)gelu_eval_any((int32_t)(int8_t)threadIdx.x, I.P);
    __syncthreads();
    if (i < n16) stream_store(gather(first), out4 + i);
    i += stride;
    for (; i < n16; i += stride) stream_store(gather(load16(i)), out4 + i);
    if (lb == 0) {
        const int64_t j = (n16 << 4) + threadIdx.x;
        if (threadIdx.x < 16 && j < n) I.out[j] = table[I.in[j]];
        if (threadIdx.x >= 32 && threadIdx.x < 32 + I.head) {     // the peeled bytes in front
            const int64_t h = (int64_t)(threadIdx.x - 32) - (int64_t)I.head;
            I.out[h] = table[I.in[h]];
        }
    }
}

// int8 -> int8, polynomial evaluated per element (no table).
template <int MODE>   // 0: general evaluation, 1: short evaluation degree 2, 2: short evaluation degree 4
__global__ void __launch_bounds__(256)
gelu_i8_direct_kernel(const uint8_t *in, uint8_t *out, int64_t n, GeluDev P)
{
    const int64_t n16 = n >> 4;
    const u32x4 *in4 = reinterpret_cast<const u32x4 *>(in);
    u32x4 *out4 = reinterpret_cast<u32x4 *>(out);
    const int64_t stride = (int64_t)gridDim.x * 256;
    auto one = [&](int32_t x) -> int32_t {
        if (MODE == 0) return gelu_eval_any(x, P);
        const int32_t q = clamp_i32(x - P.zp_in, -P.max_abs_q, P.max_abs_q);
        return gelu_eval_fast<MODE == 2>(q, P);
    };
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) {
        const u32x4 v = stream_load(in4 + i);
        u32x4 r;
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const uint32_t w = v[d];
            r[d] = pack4(one(sbyte(w, 0)), one(sbyte(w, 1)), one(sbyte(w, 2)), one(sbyte(w, 3)));
        }
        stream_store(r, out4 + i);
    }
    if (blockIdx.x == 0) {
        const int64_t i = (n16 << 4) + threadIdx.x;
        if (threadIdx.x < 16 && i < n) out[i] = (uint8_t)one((int32_t)(int8_t)in[i]);
    }
}

// Unaligned or tiny int8 tensors: one element per thread.
__global__ void __launch_bounds__(256)
gelu_i8_bytes_kernel(const uint8_t *in, uint8_t *out, int64_t n, GeluDev P)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride)
        out[i] = (uint8_t)gelu_eval_any((int32_t)(int8_t)in[i], P);
}

// int32 -> byte streaming skeleton shared by the int32 GELU and the requantization: lane i
// of a pass owns the 4 consecutive elements of 16-byte chunk i (a wavefront reads 1 KiB
// contiguous per load and writes 256 B contiguous per store).  One chunk in flight per thread
// and many resident wavefronts measured fastest on MI355X (deeper per-thread unrolling lost
// 10 %).  ALIGNED: `out` is 4-byte aligned (the host peels the `head` elements in front of
// that boundary off the tensor; the first workgroup does them too) and `in` is an int32
// pointer anywhere on the 4-byte grid: the same global_load_dwordx4 serves an input on the
// 16-byte grid and one off it.
typedef i32x4 __attribute__((aligned(4))) i32x4_a4;
template <bool ALIGNED, typename F>
IPTQ_DEV void stream_i32_to_bytes(const int32_t *in, uint8_t *out, int64_t n, int32_t head, F one)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    const int64_t tid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (ALIGNED) {
        const int64_t n4 = n >> 2;
        const i32x4_a4 *in4 = reinterpret_cast<const i32x4_a4 *>(in);
        uint32_t *out32 = reinterpret_cast<uint32_t *>(out);
        for (int64_t i = tid; i < n4; i += stride) {
            const i32x4 v = __builtin_nontemporal_load(in4 + i);
            stream_store(pack4(one(v.x), one(v.y), one(v.z), one(v.w)), out32 + i);
        }
        if (blockIdx.x == 0) {
            const int64_t i = (n4 << 2) + threadIdx.x;
            if (threadIdx.x < 4 && i < n) out[i] = (uint8_t)one(in[i]);
            if (threadIdx.x >= 32 && (int32_t)threadIdx.x < 32 + head) {   // the peeled elements in front
                const int64_t h = (int64_t)threadIdx.x - 32 - head;
                out[h] = (uint8_t)one(in[h]);
            }
        }
    } else {
        for (int64_t i = tid; i < n; i += stride) out[i] = (uint8_t)one(in[i]);
    }
}

// int32 accumulators -> int8 GELU with the requantization in front.
// MODE 0: general evaluation; 1 / 2: short evaluation of degree 2 / 4 with no or a narrow
// (pre_s >= 15) pre-requantization.
template <bool ALIGNED, int MODE>
__global__ void __launch_bounds__(256)
gelu_i32_kernel(const int32_t *in, uint8_t *out, int64_t n, int32_t head, GeluDev P)
{
    GeluDev Q = P;
    Q.zp_in = 0;
    auto one = [&](int32_t x) -> int32_t {
        if (MODE == 0) {
            if (P.pre_mode != 0) x = pre_requant_dev(x, P.pre_m, P.pre_s);
            // in - zp_in may leave 32 bits; clamping the 64-bit difference to +-max_abs_q first
            // gives the same q as the definition
            const int64_t c = (int64_t)x - (int64_t)P.zp_in;
            const int64_t lim = (int64_t)P.max_abs_q;
            const int32_t q = (int32_t)(c < -lim ? -lim : (c > lim ? lim : c));
            return gelu_eval_any(q, Q);
        }
        if (P.pre_mode == 1)     // |x * m + round| < 2^47 and pre_s >= 15: the result fits 32 bits
            x = (int32_t)(((int64_t)x * (int64_t)P.pre_m + ((int64_t)1 << (P.pre_s - 1))) >> P.pre_s);
        // a saturated difference is beyond +-max_abs_q exactly when the true one is
        const int32_t q = clamp_i32(__builtin_elementwise_sub_sat(x, P.zp_in), -P.max_abs_q, P.max_abs_q);
        return gelu_eval_fast<MODE == 2>(q, P);
    };
    stream_i32_to_bytes<ALIGNED>(in, out, n, head, one);
}

// int32 accumulators -> int8 GELU through a table.  After the requantization in front the
// centred input is clamped to [-max_abs_q, max_abs_q]; for max_abs_q <= kGelu32TableMaxQ each
// workgroup evaluates the polynomial once for every possible q with the exact formula, and an
// element costs one multiply-shift, a clamp and a byte gather from LDS.
constexpr int kGelu32TableMaxQ = 511;
constexpr int64_t kGelu32TableGridCap = 256 * 64;
template <bool ALIGNED>
__global__ void __launch_bounds__(256)
gelu_i32_table_kernel(const int32_t *in, uint8_t *out, int64_t n, int32_t head, GeluDev P)
{
    __shared__ uint8_t table[2 * kGelu32TableMaxQ + 2];
    GeluDev Q = P;
    Q.zp_in = 0;
    const int32_t lim = P.max_abs_q;
    auto one = [&](int32_t x) -> int32_t {
        if (P.pre_mode == 1)     // |x * m + round| < 2^47 and pre_s >= 15: the result fits 32 bits
            x = (int32_t)(((int64_t)x * (int64_t)P.pre_m + ((int64_t)1 << (P.pre_s - 1))) >> P.pre_s);
        else if (P.pre_mode == 2)
            x = pre_requant_dev(x, P.pre_m, P.pre_s);
        // a saturated difference is beyond +-max_abs_q exactly when the true one is
        const int32_t q = clamp_i32(__builtin_elementwise_sub_sat(x, P.zp_in), -lim, lim);
        return (int32_t)table[q + lim];
    };
    if (ALIGNED) {
        // the first chunk's load is in flight while the table is built
        const int64_t stride = (int64_t)gridDim.x * 256;
        const int64_t n4 = n >> 2;
        const i32x4_a4 *in4 = reinterpret_cast<const i32x4_a4 *>(in);
        uint32_t *out32 = reinterpret_cast<uint32_t *>(out);
        int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
        i32x4 v = {0, 0, 0, 0};
        if (i < n4) v = __builtin_nontemporal_load(in4 + i);
        for (int32_t e = threadIdx.x; e <= 2 * lim; e += 256)
            table[e] = (uint8_t)gelu_eval_any(e - lim, Q);
        __syncthreads();
        if (i < n4) stream_store(pack4(one(v.x), one(v.y), one(v.z), one(v.w)), out32 + i);
        for (i += stride; i < n4; i += stride) {
            v = __builtin_nontemporal_load(in4 + i);
            stream_store(pack4(one(v.x), one(v.y), one(v.z), one(v.w)), out32 + i);
        }
        if (blockIdx.x == 0) {
            const int64_t j = (n4 << 2) + threadIdx.x;
            if (threadIdx.x < 4 && j < n) out[j] = (uint8_t)one(in[j]);
            if (threadIdx.x >= 32 && (int32_t)threadIdx.x < 32 + head) {   // the peeled elements in front
                const int64_t h = (int64_t)threadIdx.x - 32 - head;
                out[h] = (uint8_t)one(in[h]);
            }
        }
        return;
    }
    for (int32_t e = threadIdx.x; e <= 2 * lim; e += 256)
        table[e] = (uint8_t)gelu_eval_any(e - lim, Q);
    __syncthreads();
    stream_i32_to_bytes<ALIGNED>(in, out, n, head, one);
}

// int32 -> int8 / uint8 requantization.
template <bool ALIGNED>
__global__ void __launch_bounds__(256)
requant_kernel(const int32_t *in, uint8_t *out, int64_t n, int32_t head, DyadicDev P)
{
    auto one = [&](int32_t x) -> int32_t {
        return P.s >= 16 ? requant_dev<true>(x, P.m, P.s, P.zp, P.qmin, P.qmax)
                         : requant_dev<false>(x, P.m, P.s, P.zp, P.qmin, P.qmax);
    };
    stream_i32_to_bytes<ALIGNED>(in, out, n, head, one);
}

// ---------------------------------------------------------------------------------------
// Host-side dispatch.  Grid: enough workgroups to fill 256 compute units several times
// over, capped by the amount of work.

static unsigned grid_for(int64_t work_items, int per_block, int64_t cap = 256 * 16)
{
    int64_t g = (work_items + per_block - 1) / per_block;
    if (g > cap) g = cap;
    if (g < 1) g = 1;
    return (unsigned)g;
}

hipError_t gelu_i8_dispatch(const GeluCall *calls, int n_calls, hipStream_t stream)
{
    GeluBatch B;
    B.n_items = 0;
    unsigned total_wgs = 0;
    auto flush = [&]() {
        if (B.n_items == 0) return;
        hipLaunchKernelGGL(gelu_i8_table_kernel, dim3(total_wgs), dim3(256), 0, stream, B);
        B.n_items = 0;
        total_wgs = 0;
    };
    for (int c = 0; c < n_calls; ++c) {
        const GeluCall &g = calls[c];
        if (g.n == 0) continue;
        const uint8_t *uin = reinterpret_cast<const uint8_t *>(g.in);
        uint8_t *uout = reinterpret_cast<uint8_t *>(g.out);
        const bool aligned = ((reinterpret_cast<uintptr_t>(g.in) | reinterpret_cast<uintptr_t>(g.out)) & 15) == 0;
        // bytes in front of the output's first 16-byte boundary
        const uint32_t head = (uint32_t)((0 - reinterpret_cast<uintptr_t>(g.out)) & 15);
        if (!aligned && (g.force_direct || g.n < 64)) {
            hipLaunchKernelGGL(gelu_i8_bytes_kernel, dim3(grid_for(g.n, 256)), dim3(256), 0, stream,
                               uin, uout, g.n, g.P);
        } else if (g.force_direct) {
            const dim3 grid(grid_for(g.n >> 4, 256, 256 * 64));
            if (!g.P.fast)
                hipLaunchKernelGGL(gelu_i8_direct_kernel<0>, grid, dim3(256), 0, stream, uin, uout, g.n, g.P);
            else if (!g.P.quartic)
                hipLaunchKernelGGL(gelu_i8_direct_kernel<1>, grid, dim3(256), 0, stream, uin, uout, g.n, g.P);
            else
                hipLaunchKernelGGL(gelu_i8_direct_kernel<2>, grid, dim3(256), 0, stream, uin, uout, g.n, g.P);
        } else {
            if (B.n_items == kGeluBatchMax) flush();
            GeluItem &it = B.item[B.n_items++];
            it.in = uin + head; it.out = uout + head; it.n = g.n - head; it.P = g.P;
            it.head = head;
            it.first_wg = total_wgs;
            it.n_wgs = grid_for(it.n >> 4, 256, kGeluTableGridCap);
            total_wgs += it.n_wgs;
        }
    }
    flush();
    return hipGetLastError();
}

// The vector path of the int32-input kernels wants a 4-byte aligned output: the elements in
// front of that boundary are peeled off (the kernel's first workgroup does them), the input
// follows wherever that leaves it on its 4-byte grid.  Calls too short for that stream bytes.
static bool peel_to_dword_out(const int32_t *&in, uint8_t *&out, int64_t &n, int32_t *head)
{
    *head = (int32_t)((0 - reinterpret_cast<uintptr_t>(out)) & 3);
    if ((reinterpret_cast<uintptr_t>(in) & 3) != 0 || n < 64) return false;
    in += *head; out += *head; n -= *head;
    return true;
}

hipError_t gelu_i32_dispatch(const int32_t *in, int8_t *out, int64_t n, const GeluDev &P,
                             bool force_direct, hipStream_t stream)
{
    uint8_t *uout = reinterpret_cast<uint8_t *>(out);
    int32_t head = 0;
    const bool aligned = peel_to_dword_out(in, uout, n, &head);
    const int mode = (P.fast && P.pre_mode != 2) ? (P.quartic ? 2 : 1) : 0;
    const bool table = !force_direct && P.max_abs_q <= kGelu32TableMaxQ;
    if (aligned) {
        const dim3 grid(grid_for(n >> 2, 256, 256 * 64)), block(256);
        if (table)
            hipLaunchKernelGGL(gelu_i32_table_kernel<true>, dim3(grid_for(n >> 2, 256, kGelu32TableGridCap)),
                               block, 0, stream, in, uout, n, head, P);
        else if (mode == 0) hipLaunchKernelGGL((gelu_i32_kernel<true, 0>), grid, block, 0, stream, in, uout, n, head, P);
        else if (mode == 1) hipLaunchKernelGGL((gelu_i32_kernel<true, 1>), grid, block, 0, stream, in, uout, n, head, P);
        else hipLaunchKernelGGL((gelu_i32_kernel<true, 2>), grid, block, 0, stream, in, uout, n, head, P);
    } else {
        const dim3 grid(grid_for(n, 256)), block(256);
        if (table) hipLaunchKernelGGL(gelu_i32_table_kernel<false>, grid, block, 0, stream, in, uout, n, 0, P);
        else if (mode == 0) hipLaunchKernelGGL((gelu_i32_kernel<false, 0>), grid, block, 0, stream, in, uout, n, 0, P);
        else if (mode == 1) hipLaunchKernelGGL((gelu_i32_kernel<false, 1>), grid, block, 0, stream, in, uout, n, 0, P);
        else hipLaunchKernelGGL((gelu_i32_kernel<false, 2>), grid, block, 0, stream, in, uout, n, 0, P);
    }
    return hipGetLastError();
}

hipError_t requant_dispatch(const int32_t *in, void *out, int64_t n, const DyadicDev &P,
                            hipStream_t stream)
{
    uint8_t *uout = reinterpret_cast<uint8_t *>(out);
    int32_t head = 0;
    // Up to about 100 MB one resident generation of workgroups (8 per compute unit) that loop is
    // faster than many short-lived ones (kernel-trace durations: 24.6 MB 5.8 against 6.7 us,
    // 49 MB 9.4 against 10.7, 98 MB 16.7 against 18.2); from 200 MB on the order reverses
    // (298 MB: 48.8 against 47.3 us).
    const int64_t cap = n <= 25 * 1000 * 1000 ? 256 * 8 : 256 * 64;
    if (peel_to_dword_out(in, uout, n, &head))
        hipLaunchKernelGGL(requant_kernel<true>, dim3(grid_for(n >> 2, 256, cap)), dim3(256), 0, stream, in,
                           uout, n, head, P);
    else
        hipLaunchKernelGGL(requant_kernel<false>, dim3(grid_for(n, 256)), dim3(256), 0, stream, in, uout,
                           n, 0, P);
    return hipGetLastError();
}

}  // namespace iptq
