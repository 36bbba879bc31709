// One-wavefront-per-row softmax kernel, up to 20 passes of 64 blocks (rows of up to 5117 scores).
#include "softmax_wide.h"

namespace iptq {
void wide_launch_s20(const WideArgs &A, int mode, int post_mode, dim3 grid, hipStream_t stream)
{
    wide_launch_s<20>(A, mode, post_mode, grid, stream);
}
}
