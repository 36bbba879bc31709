// One-wavefront-per-row softmax kernel, up to 8 passes of 64 blocks (rows of up to 2045 scores).
#include "softmax_wide.h"

namespace iptq {
void wide_launch_s8(const WideArgs &A, int mode, int post_mode, dim3 grid, hipStream_t stream)
{
    wide_launch_s<8>(A, mode, post_mode, grid, stream);
}
}
