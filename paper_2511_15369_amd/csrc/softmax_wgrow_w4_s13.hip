// One-workgroup-per-row softmax kernel, 4 wavefronts, up to 13 passes (rows of up to 13309 scores).
#include "softmax_wgrow.h"

namespace iptq {
void wgrow_launch_w4_s13(const WideArgs &A, int mode, int post_mode, dim3 grid, hipStream_t stream)
{
    wgrow_launch_ws<4, 13>(A, mode, post_mode, grid, stream);
}
}
