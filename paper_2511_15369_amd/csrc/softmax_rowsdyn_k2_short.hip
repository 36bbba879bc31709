// Run-time-row-length softmax slab kernel, 2 lanes per row, 1 to 4 blocks per lane.
#include "softmax_rowsdyn.h"

namespace iptq {
bool rowsdyn_launch_k2_short(const DynArgs &A, int slots, int mode, dim3 grid, dim3 block, size_t lds, hipStream_t stream)
{
    switch (slots) {
    IPTQ_ROWSDYN_CASE(2, 1)
    IPTQ_ROWSDYN_CASE(2, 2)
    IPTQ_ROWSDYN_CASE(2, 3)
    IPTQ_ROWSDYN_CASE(2, 4)
    default: return false;
    }
}
}  // namespace iptq
