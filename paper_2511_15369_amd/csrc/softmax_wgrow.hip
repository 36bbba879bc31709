// Host side of the one-workgroup-per-row softmax kernel (softmax_wgrow.h).
#include <hip/hip_runtime.h>

#include "softmax_wgrow.h"

namespace iptq {

// Wavefronts per workgroup and pass count for a row length (exactly the passes a row needs at its
// worst alignment: the kernels rely on it); false beyond 40957 scores.  Up to 13 passes keep a
// lane within 128 registers, so two workgroups share a compute unit and one loads while the
// other computes (66-78 % of the HBM roofline); the 14 to 20 passes that 8 wavefronts would
// need beyond 26618 scores leave one workgroup per compute unit, and so do 16 wavefronts
// (both 46-50 %; 16 wavefronts compile faster).
bool wgrow_geometry(int32_t cols, int *waves, int *slots, bool off_grid)
{
    // off_grid: as for wide_geometry
    const int nb_max = (off_grid || cols % 2 != 0) ? (cols + 3 + 3) / 4 : ((cols % 4 == 0) ? cols / 4 : (cols + 2 + 3) / 4);
    int w = 4;
    if ((nb_max + 255) / 256 > 13) w = 8;
    if ((nb_max + 511) / 512 > 13) w = 16;
    const int n = (nb_max + 64 * w - 1) / (64 * w);
    if (n > (w == 16 ? 10 : 13)) return false;
    *waves = w;
    *slots = n;
    return true;
}

// Every row of one call if the call qualifies (same conditions as softmax_wide_launch).
hipError_t softmax_wgrow_launch(const SoftmaxCall &c, int32_t cols, int post_mode, int64_t *done,
                                hipStream_t stream)
{
    *done = 0;
    int waves = 0, slots = 0;
    // The tensor may start anywhere on the 4-byte grid (rows are addressed on the 16-byte grid
    // below it) and the output anywhere; the additive table is indexed block by block and needs
    // both tensors on the 16-byte grid.
    const uintptr_t sa = reinterpret_cast<uintptr_t>(c.scores);
    const int base_off = (int)((sa & 15) >> 2);
    if ((sa & 3) != 0) return hipSuccess;
    if (!wgrow_geometry(cols, &waves, &slots, base_off != 0)) return hipSuccess;
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
    const dim3 grid((unsigned)rows);                  // one workgroup per row, exactly
    const int mode = c.P.mode16;
    bool launched;
    if (waves == 4) launched = slots <= 9 ? wgrow_launch_w4_lo(A, slots, mode, grid, stream) : wgrow_launch_w4_hi(A, slots, mode, grid, stream);
    else if (waves == 8) launched = slots <= 10 ? wgrow_launch_w8_lo(A, slots, mode, grid, stream) : wgrow_launch_w8_hi(A, slots, mode, grid, stream);
    else launched = wgrow_launch_w16(A, slots, mode, grid, stream);
    if (!launched) return hipSuccess;
    *done = rows;
    return hipGetLastError();
}

}  // namespace iptq
