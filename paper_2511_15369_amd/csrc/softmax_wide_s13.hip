// One-wavefront-per-row softmax kernel, up to 13 passes of 64 blocks (rows of up to 3325 scores).
#include "softmax_wide.h"

namespace iptq {
void wide_launch_s13(const WideArgs &A, int mode, int post_mode, dim3 grid, hipStream_t stream)
{
    wide_launch_s<13>(A, mode, post_mode, grid, stream);
}
}
