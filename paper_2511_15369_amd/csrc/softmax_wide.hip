// Host side of the one-wavefront-per-row softmax kernel (softmax_wide.h).
#include <hip/hip_runtime.h>

#include "softmax_wide.h"

namespace iptq {

// Passes of 64 blocks a row of `cols` scores needs at its worst alignment (exactly: the kernel
// compiled for that count serves it and relies on it).  Returns false beyond 16 passes (rows of
// more than 4093 scores, 4096 if a multiple of 4): with more registers per lane than that a
// workgroup per row is faster (softmax_wgrow.h).
bool wide_geometry(int32_t cols, int *passes, int *slots, bool off_grid)
{
    // off_grid: the tensor itself starts off the 16-byte grid, so a row can start at any element of
    // a block whatever the row length
    const int nb_max = (off_grid || cols % 2 != 0) ? (cols + 3 + 3) / 4 : ((cols % 4 == 0) ? cols / 4 : (cols + 2 + 3) / 4);
    const int n = (nb_max + 63) / 64;
    if (n > 16) return false;
    *passes = n;
    *slots = n;
    return true;
}

// Every row of one call if the call qualifies (rows of up to 16 passes, pointers as checked
// below); *done receives the number of rows served (0: not served, nothing enqueued).
hipError_t softmax_wide_launch(const SoftmaxCall &c, int32_t cols, int post_mode, int64_t *done,
                               hipStream_t stream)
{
    *done = 0;
    int n = 0, slots = 0;
    // The tensor may start anywhere on the 4-byte grid (rows are addressed on the 16-byte grid
    // below it) and the output anywhere; the additive table is indexed block by block and needs
    // both tensors on the 16-byte grid.
    const uintptr_t sa = reinterpret_cast<uintptr_t>(c.scores);
    const int base_off = (int)((sa & 15) >> 2);
    if ((sa & 3) != 0) return hipSuccess;
    if (!wide_geometry(cols, &n, &slots, base_off != 0)) return hipSuccess;
    const bool has_bias = c.bias != nullptr;
    const bool bias_ok = !has_bias || (base_off == 0 && (reinterpret_cast<uintptr_t>(c.bias) & 15) == 0 &&
                                       ((int64_t)c.P.bias_period_rows * cols) % 4 == 0);
    if (!bias_ok) return hipSuccess;
    // A tensor that ends off the 16-byte grid: the kernel loads the last row's final block
    // element by element, which takes rows of at least 8 scores (a whole block before it).
    const int cut_el = (int)((base_off + c.rows * cols) & 3);
    if (c.rows <= 0 || (cut_el != 0 && cols < 8)) return hipSuccess;
    const int64_t rows = c.rows;
    WideArgs A;
    A.scores = c.scores - base_off; A.bias = c.bias; A.out = c.out - base_off; A.base_off = base_off; A.rows = rows; A.cols = cols; A.post_mode = post_mode; A.P = c.P;
    A.cut_el = cut_el;
    const dim3 grid((unsigned)((rows + 3) / 4));
    const int mode = c.P.mode16;
    const bool launched = n <= 6 ? wide_launch_p1_6(A, n, mode, grid, stream)
                        : n <= 10 ? wide_launch_p7_10(A, n, mode, grid, stream)
                        : n <= 13 ? wide_launch_p11_13(A, n, mode, grid, stream)
                                  : wide_launch_p14_16(A, n, mode, grid, stream);
    if (!launched) return hipSuccess;
    *done = rows;
    return hipGetLastError();
}

}  // namespace iptq
