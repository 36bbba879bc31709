// Integer-only device helpers shared by the gfx950 kernels.  Nothing in this file may
// compile to a floating-point instruction: no '/' or '%' on run-time values (the compiler
// lowers those through v_rcp_f32), no float types.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#define IPTQ_DEV __device__ __forceinline__
#define IPTQ_HD __host__ __device__ inline

namespace iptq {

constexpr int32_t kI32Min = (int32_t)0x80000000;

typedef int32_t i32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Streaming accesses: every byte is touched once, so the loads and stores carry the
// non-temporal hint and do not displace reusable lines (the bias table) from the caches.
template <typename T>
__device__ __forceinline__ T stream_load(const T *p)
{
    return __builtin_nontemporal_load(p);
}
template <typename T>
__device__ __forceinline__ void stream_store(T v, T *p)
{
    __builtin_nontemporal_store(v, p);
}

// 16-byte and 4-byte accesses at addresses that are only as aligned as their elements: a
// tensor that is a view into a larger one can start anywhere on its element grid, and
// global_load_dwordx4 / global_store_dwordx4 take any address on this part.  The pointer
// types say so; the instructions are the ones an aligned access compiles to.
typedef i32x4 __attribute__((aligned(4))) i32x4_a4;
typedef u32x4 __attribute__((aligned(1))) u32x4_a1;
typedef uint32_t __attribute__((aligned(1))) u32_a1;
__device__ __forceinline__ i32x4 stream_load_i32x4(const int32_t *p)
{
    return __builtin_nontemporal_load(reinterpret_cast<const i32x4_a4 *>(p));
}
__device__ __forceinline__ i32x4 load_i32x4(const int32_t *p)
{
    return *reinterpret_cast<const i32x4_a4 *>(p);
}
// The same at a byte offset below 2^32 from a wavefront-uniform base: compiles to the form with a
// scalar base and a 32-bit vector offset (no 64-bit address arithmetic per load).
__device__ __forceinline__ i32x4 load_i32x4_at(const int32_t *base, uint32_t byte_offset)
{
    return *reinterpret_cast<const i32x4_a4 *>(reinterpret_cast<const char *>(base) + byte_offset);
}
__device__ __forceinline__ void stream_store_bytes16(u32x4 v, uint8_t *p)
{
    __builtin_nontemporal_store(v, reinterpret_cast<u32x4_a1 *>(p));
}
__device__ __forceinline__ void stream_store_bytes4(uint32_t v, uint8_t *p)
{
    __builtin_nontemporal_store(v, reinterpret_cast<u32_a1 *>(p));
}

IPTQ_HD uint32_t mulhi_u32(uint32_t a, uint32_t b)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return __umulhi(a, b);
#else
    return (uint32_t)(((uint64_t)a * b) >> 32);
#endif
}

IPTQ_HD int clz_u32(uint32_t v)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return __clz((int)v);
#else
    return v ? __builtin_clz(v) : 32;
#endif
}

// floor(2^m_bits / sigma) for 1 <= sigma <= 2^m_bits, 1 <= m_bits <= 31, without a divide
// instruction: normalise sigma to y in [2^31, 2^32), run three Newton steps on the Q31
// reciprocal (each keeps the estimate at or below the true value), scale back and finish
// with an exact remainder correction.  sigma == 0 returns 0.
IPTQ_HD uint32_t floor_pow2_div(int m_bits, uint32_t sigma)
{
    if (sigma == 0) return 0;
    const int k = clz_u32(sigma);
    const uint32_t y = sigma << k;                    // Y = y / 2^32 in [0.5, 1)
    // X0 = 48/17 - 32/17 Y in Q30, then to Q31: relative error below 1/17, X0 < 1/Y
    uint32_t r = (3031741620u - mulhi_u32(y, 2021161080u)) << 1;
    for (int it = 0; it < 3; ++it) {
        const uint32_t t = mulhi_u32(y, r);           // Y X in Q31, at most 2^31
        const uint32_t u = 0u - t;                    // (2 - Y X) in Q31
        r = mulhi_u32(r, u) << 1;                     // X (2 - Y X) in Q31, rounded down
    }
    // 2^m / sigma = (2^63 / y) * 2^(m + k - 63), r ~ 2^63 / y
    const int sh = 63 - m_bits - k;                   // 1 <= sh <= 32
    uint32_t f = sh >= 32 ? 0u : (r >> sh);
    uint32_t rem = (1u << m_bits) - f * sigma;        // exact: f <= true quotient
    while (rem >= sigma) { rem -= sigma; ++f; }
    return f;
}

// clamp(rshr_round(x * m, s) + zp, qmin, qmax) for |x| < 2^31, |m| < 2^15, 0 <= s <= 62.
// NARROW (s >= 16): the shifted value fits 32 bits.
template <bool NARROW>
IPTQ_DEV int32_t requant_dev(int32_t x, int32_t m, int32_t s, int32_t zp, int32_t qmin, int32_t qmax)
{
    const int64_t rnd = s > 0 ? ((int64_t)1 << (s - 1)) : 0;
    const int64_t v = (int64_t)x * (int64_t)m + rnd;
    if (NARROW) {
        const int32_t r = (int32_t)(v >> s) + zp;
        return min(max(r, qmin), qmax);
    } else {
        int64_t r = (v >> s) + (int64_t)zp;
        r = r < (int64_t)qmin ? (int64_t)qmin : r;
        r = r > (int64_t)qmax ? (int64_t)qmax : r;
        return (int32_t)r;
    }
}

// sat32(rshr_round(x * m, s)), 1 <= m < 2^15, 0 <= s <= 62
IPTQ_DEV int32_t pre_requant_dev(int32_t x, int32_t m, int32_t s)
{
    const int64_t rnd = s > 0 ? ((int64_t)1 << (s - 1)) : 0;
    int64_t v = ((int64_t)x * (int64_t)m + rnd) >> s;
    v = v < (int64_t)INT32_MIN ? (int64_t)INT32_MIN : v;
    v = v > (int64_t)INT32_MAX ? (int64_t)INT32_MAX : v;
    return (int32_t)v;
}

// clamp(v, lo, hi) for lo <= hi in one instruction (the compiler cannot prove lo <= hi for
// run-time bounds and would emit a max and a min)
IPTQ_DEV int32_t clamp_i32(int32_t v, int32_t lo, int32_t hi)
{
    int32_t r;
    asm("v_med3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(v), "v"(lo), "v"(hi));
    return r;
}

// Every launch starts with a cold scalar cache, and a kernel that reads its arguments in dependent
// steps (which problem of the batch, then that problem's sizes, then its table constants) waits
// for memory once per step before it can issue its first load.  This touches the first BYTES of
// the kernel-argument segment at once, one load per 64-byte line, so that one wait covers them
// all and the steps that follow hit in the cache.
template <int BYTES>
IPTQ_DEV void touch_kernel_arguments()
{
    typedef const __attribute__((address_space(4))) uint32_t *ArgWords;
    ArgWords ka = (ArgWords)__builtin_amdgcn_kernarg_segment_ptr();
    static_assert(BYTES > 0 && BYTES <= 512, "at most eight lines");
    constexpr int LINES = (BYTES + 63) / 64;
    uint32_t t[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < LINES; ++i) t[i] = ka[16 * i];
    asm volatile("" ::"s"(t[0]), "s"(t[1]), "s"(t[2]), "s"(t[3]), "s"(t[4]), "s"(t[5]), "s"(t[6]), "s"(t[7]));
}

// (mask & a) | (~mask & b) in one instruction (written out, the compiler turns a select on a
// single bit into a test, a compare and a conditional move per element)
IPTQ_DEV int32_t select_bits_i32(uint32_t mask, int32_t a, int32_t b)
{
    int32_t r;
    asm("v_bfi_b32 %0, %1, %2, %3" : "=v"(r) : "v"(mask), "v"(a), "v"(b));
    return r;
}

IPTQ_DEV int32_t sat_add_i32(int32_t a, int32_t b)
{
    return __builtin_elementwise_add_sat(a, b);
}

// score + t for one entry t of an additive table (relative-position bias, window mask): minus
// infinity if either is, else the saturating sum.
IPTQ_DEV int32_t add_table_entry(int32_t x, int32_t t)
{
    const int32_t s = sat_add_i32(x, t);
    return min(x, t) == kI32Min ? kI32Min : s;
}

IPTQ_DEV i32x4 add_table_chunk(i32x4 v, i32x4 t)
{
    v.x = add_table_entry(v.x, t.x);
    v.y = add_table_entry(v.y, t.y);
    v.z = add_table_entry(v.z, t.z);
    v.w = add_table_entry(v.w, t.w);
    return v;
}

// ---- cross-lane exchange on the DPP path (no LDS traffic) -----------------------------
// DPP control words: quad_perm [1,0,3,2] = 0xB1, quad_perm [2,3,0,1] = 0x4E,
// row_half_mirror = 0x141, row_mirror = 0x140.
template <int CTRL>
IPTQ_DEV int32_t dpp_i32(int32_t v)
{
    return __builtin_amdgcn_update_dpp(v, v, CTRL, 0xF, 0xF, false);
}

// All-reduce over aligned groups of K lanes (K a power of two up to 64); every lane gets the
// result.  Up to 16 lanes stay on the DPP path; 32 and 64 add steps through the permute network.
template <int K>
IPTQ_DEV int32_t group_max_i32(int32_t v)
{
    if (K >= 2) v = max(v, dpp_i32<0xB1>(v));
    if (K >= 4) v = max(v, dpp_i32<0x4E>(v));
    if (K >= 8) v = max(v, dpp_i32<0x141>(v));
    if (K >= 16) v = max(v, dpp_i32<0x140>(v));
    if (K >= 32) v = max(v, __shfl_xor(v, 16));
    if (K >= 64) v = max(v, __shfl_xor(v, 32));
    return v;
}

template <int K>
IPTQ_DEV uint32_t group_sum_u32(uint32_t v)
{
    if (K >= 2) v += (uint32_t)dpp_i32<0xB1>((int32_t)v);
    if (K >= 4) v += (uint32_t)dpp_i32<0x4E>((int32_t)v);
    if (K >= 8) v += (uint32_t)dpp_i32<0x141>((int32_t)v);
    if (K >= 16) v += (uint32_t)dpp_i32<0x140>((int32_t)v);
    if (K >= 32) v += (uint32_t)__shfl_xor((int32_t)v, 16);
    if (K >= 64) v += (uint32_t)__shfl_xor((int32_t)v, 32);
    return v;
}

// Full 64-lane all-reduce: the 16-lane DPP rows first, then across rows through the
// permute network.
IPTQ_DEV int32_t wave_max_i32(int32_t v)
{
    v = group_max_i32<16>(v);
    v = max(v, __shfl_xor(v, 16));
    v = max(v, __shfl_xor(v, 32));
    return v;
}

IPTQ_DEV uint32_t wave_sum_u32(uint32_t v)
{
    v = group_sum_u32<16>(v);
    v += (uint32_t)__shfl_xor((int32_t)v, 16);
    v += (uint32_t)__shfl_xor((int32_t)v, 32);
    return v;
}

// Orders this wavefront's LDS accesses: what its lanes wrote before is visible to its
// lanes after.  LDS executes a wavefront's instructions in issue order, so this only has
// to stop the compiler from moving accesses across it.
IPTQ_DEV void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

}  // namespace iptq
