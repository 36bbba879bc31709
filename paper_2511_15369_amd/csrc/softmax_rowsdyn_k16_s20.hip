// Run-time-row-length softmax slab kernel, 16 lanes per row, up to 20 blocks per lane.
#include "softmax_rowsdyn.h"

namespace iptq {
void rowsdyn_launch_k16_s20(const DynArgs &A, int mode, int post_mode, dim3 grid, dim3 block, size_t lds,
                            hipStream_t stream)
{
    rowsdyn_launch_ks<16, 20>(A, mode, post_mode, grid, block, lds, stream);
}
}
