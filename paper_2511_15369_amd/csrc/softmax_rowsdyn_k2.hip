// Run-time-row-length softmax slab kernel, 2 lanes per row, 5 to 8 blocks per lane.
#include "softmax_rowsdyn.h"

namespace iptq {
bool rowsdyn_launch_k2(const DynArgs &A, int slots, int mode, dim3 grid, dim3 block, size_t lds, hipStream_t stream)
{
    switch (slots) {
    IPTQ_ROWSDYN_CASE(2, 5)
    IPTQ_ROWSDYN_CASE(2, 6)
    IPTQ_ROWSDYN_CASE(2, 7)
    IPTQ_ROWSDYN_CASE(2, 8)
    default: return false;
    }
}
}  // namespace iptq
