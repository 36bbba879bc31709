// Run-time-row-length softmax slab kernel, 4 lanes per row, 5 to 8 blocks per lane.
#include "softmax_rowsdyn.h"

namespace iptq {
bool rowsdyn_launch_k4(const DynArgs &A, int slots, int mode, dim3 grid, dim3 block, size_t lds, hipStream_t stream)
{
    switch (slots) {
    IPTQ_ROWSDYN_CASE(4, 5)
    IPTQ_ROWSDYN_CASE(4, 6)
    IPTQ_ROWSDYN_CASE(4, 7)
    IPTQ_ROWSDYN_CASE(4, 8)
    default: return false;
    }
}
}  // namespace iptq
