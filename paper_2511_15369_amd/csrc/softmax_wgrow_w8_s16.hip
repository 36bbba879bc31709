// One-workgroup-per-row softmax kernel, 8 wavefronts, up to 16 passes (rows of up to 32765 scores).
#include "softmax_wgrow.h"

namespace iptq {
void wgrow_launch_w8_s16(const WideArgs &A, int mode, int post_mode, dim3 grid, hipStream_t stream)
{
    wgrow_launch_ws<8, 16>(A, mode, post_mode, grid, stream);
}
}
