// One-workgroup-per-row softmax kernel, 4 wavefronts, up to 20 passes (rows of up to 20477 scores).
#include "softmax_wgrow.h"

namespace iptq {
void wgrow_launch_w4_s20(const WideArgs &A, int mode, int post_mode, dim3 grid, hipStream_t stream)
{
    wgrow_launch_ws<4, 20>(A, mode, post_mode, grid, stream);
}
}
