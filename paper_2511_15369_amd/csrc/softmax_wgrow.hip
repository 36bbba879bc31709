// Host side of the one-workgroup-per-row softmax kernel (softmax_wgrow.h).
#include <hip/hip_runtime.h>

#include "softmax_wgrow.h"

namespace iptq {

// Wavefronts per workgroup and compiled pass count for a row length; false beyond 40957 scores.
bool wgrow_geometry(int32_t cols, int *waves, int *slots)
{
    const int nb_max = (cols % 4 == 0) ? cols / 4 : ((cols % 2 == 0) ? (cols + 2 + 3) / 4 : (cols + 3 + 3) / 4);
    const int n4 = (nb_max + 255) / 256, n8 = (nb_max + 511) / 512;
    if (n4 <= 13) { *waves = 4; *slots = 13; }
    else if (n4 <= 20) { *waves = 4; *slots = 20; }
    else if (n8 <= 16) { *waves = 8; *slots = 16; }
    else if (n8 <= 20) { *waves = 8; *slots = 20; }
    else return false;
    return true;
}

// Most rows of one call if the call qualifies (same conditions as softmax_wide_launch).
hipError_t softmax_wgrow_launch(const SoftmaxCall &c, int32_t cols, int post_mode, int64_t *done,
                                hipStream_t stream)
{
    *done = 0;
    int waves = 0, slots = 0;
    if (!wgrow_geometry(cols, &waves, &slots)) return hipSuccess;
    const bool has_bias = c.bias != nullptr;
    const bool aligned = ((reinterpret_cast<uintptr_t>(c.scores) | reinterpret_cast<uintptr_t>(c.out)) & 15) == 0;
    const bool bias_ok = !has_bias || ((reinterpret_cast<uintptr_t>(c.bias) & 15) == 0 &&
                                       ((int64_t)c.P.bias_period_rows * cols) % 4 == 0);
    if (!aligned || !bias_ok) return hipSuccess;
    const int64_t rows = ((c.rows * cols) % 4 == 0) ? c.rows : c.rows - 1;
    if (rows <= 0) return hipSuccess;
    WideArgs A;
    A.scores = c.scores; A.bias = c.bias; A.out = c.out; A.rows = rows; A.cols = cols; A.P = c.P;
    const dim3 grid((unsigned)rows);                  // one workgroup per row, exactly
    const int mode = c.P.mode16;
    if (waves == 4 && slots == 13) wgrow_launch_w4_s13(A, mode, post_mode, grid, stream);
    else if (waves == 4) wgrow_launch_w4_s20(A, mode, post_mode, grid, stream);
    else if (slots == 16) wgrow_launch_w8_s16(A, mode, post_mode, grid, stream);
    else wgrow_launch_w8_s20(A, mode, post_mode, grid, stream);
    *done = rows;
    return hipGetLastError();
}

}  // namespace iptq
