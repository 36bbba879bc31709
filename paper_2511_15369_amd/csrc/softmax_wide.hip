// Host side of the one-wavefront-per-row softmax kernel (softmax_wide.h).
#include <hip/hip_runtime.h>

#include "softmax_wide.h"

namespace iptq {

// Passes of 64 blocks a row of `cols` scores needs at its worst alignment, and the compiled
// pass count that serves it.  Returns false beyond 16 passes (rows of more than 4093 scores):
// with more registers per lane than that a workgroup per row is faster (softmax_wgrow.h;
// 5117 columns: 63 % against 55 % of the HBM roofline).
bool wide_geometry(int32_t cols, int *passes, int *slots)
{
    const int nb_max = (cols % 4 == 0) ? cols / 4 : ((cols % 2 == 0) ? (cols + 2 + 3) / 4 : (cols + 3 + 3) / 4);
    const int n = (nb_max + 63) / 64;
    if (n > 16) return false;
    *passes = n;
    *slots = n <= 8 ? 8 : (n <= 13 ? 13 : 16);
    return true;
}

// Most rows of one call if the call qualifies: rows of up to 4093 scores, 16-byte aligned
// tensors.  When the tensor does not end on a 16-byte boundary its last row is left out (its
// final block would reach beyond the tensor); *done receives the number of leading rows served.
hipError_t softmax_wide_launch(const SoftmaxCall &c, int32_t cols, int post_mode, int64_t *done,
                               hipStream_t stream)
{
    *done = 0;
    int n = 0, slots = 0;
    if (!wide_geometry(cols, &n, &slots)) return hipSuccess;
    const bool has_bias = c.bias != nullptr;
    const bool aligned = ((reinterpret_cast<uintptr_t>(c.scores) | reinterpret_cast<uintptr_t>(c.out)) & 15) == 0;
    const bool bias_ok = !has_bias || ((reinterpret_cast<uintptr_t>(c.bias) & 15) == 0 &&
                                       ((int64_t)c.P.bias_period_rows * cols) % 4 == 0);
    if (!aligned || !bias_ok) return hipSuccess;
    const int64_t rows = ((c.rows * cols) % 4 == 0) ? c.rows : c.rows - 1;
    if (rows <= 0) return hipSuccess;
    WideArgs A;
    A.scores = c.scores; A.bias = c.bias; A.out = c.out; A.rows = rows; A.cols = cols; A.P = c.P;
    const dim3 grid((unsigned)((rows + 3) / 4));
    const int mode = c.P.mode16;
    if (slots == 8) wide_launch_s8(A, mode, post_mode, grid, stream);
    else if (slots == 13) wide_launch_s13(A, mode, post_mode, grid, stream);
    else wide_launch_s16(A, mode, post_mode, grid, stream);
    *done = rows;
    return hipGetLastError();
}

}  // namespace iptq
