// Launch entry points of the kernel translation units (host side).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "plan.h"

namespace iptq {

// One softmax problem: rows x cols scores -> bytes, validated parameters.
struct SoftmaxCall {
    const int32_t *scores;
    const int32_t *bias;
    const int32_t *mask;  // per-window mask or nullptr (its shape is in P)
    const uint64_t *mask_bits;   // or the same mask one bit per key, ceil(cols / 64) words per query
    uint8_t *out;
    int64_t rows;
    int out_bits;
    int algo;            // IPTQ_ALGO_*
    SoftmaxDev P;
};
// One int8 GELU problem.
struct GeluCall {
    const int8_t *in;
    int8_t *out;
    int64_t n;
    bool force_direct;
    GeluDev P;
};

hipError_t softmax_dispatch(const SoftmaxCall *calls, int n_calls, int32_t cols, hipStream_t stream);
// Register-resident slab kernel with a run-time row length: every row of one call, or none
// (*done == 0) if the row is too long or the pointers do not qualify.
hipError_t softmax_rowsdyn_launch(const SoftmaxCall &c, int32_t cols, int post_mode, int64_t *done,
                                  hipStream_t stream);
// One wavefront per row, row in registers, no LDS staging (rows of up to 4093 scores at any
// alignment, 4096 if a multiple of 4): every row of one call, or none.
hipError_t softmax_wide_launch(const SoftmaxCall &c, int32_t cols, int post_mode, int64_t *done,
                               hipStream_t stream);
// One workgroup per row, row in the workgroup's registers (rows of up to 40957 scores).
hipError_t softmax_wgrow_launch(const SoftmaxCall &c, int32_t cols, int post_mode, int64_t *done,
                                hipStream_t stream);
// Host-side layout choices of the run-time-row-length kernels (false: the kernel does not
// serve that row length).
bool softmax_rows_compiled(int32_t cols);         // a kernel with this row length compiled in exists
bool rowsdyn_geometry(int32_t cols, int *lanes, int *slots);
bool wide_geometry(int32_t cols, int *passes, int *slots, bool off_grid = false);
bool wgrow_geometry(int32_t cols, int *waves, int *slots, bool off_grid = false);
hipError_t gelu_i8_dispatch(const GeluCall *calls, int n_calls, hipStream_t stream);
hipError_t gelu_i32_dispatch(const int32_t *in, int8_t *out, int64_t n, const GeluDev &P,
                             bool force_direct, hipStream_t stream);
// [n_windows, cols, cols] int32 -> [n_windows, cols, ceil(cols / 64)] words, bit k set where the entry is INT32_MIN
hipError_t pack_window_mask_dispatch(const int32_t *mask, int64_t n_queries, int32_t cols, uint64_t *bits,
                                     hipStream_t stream);
hipError_t requant_dispatch(const int32_t *in, void *out, int64_t n, const DyadicDev &P,
                            hipStream_t stream);

}  // namespace iptq
