// Run-time-row-length softmax slab kernel, 1 lane per row (rows of up to 29 scores), 1 to 8 blocks per lane.
#include "softmax_rowsdyn.h"

namespace iptq {
bool rowsdyn_launch_k1(const DynArgs &A, int slots, int mode, dim3 grid, dim3 block, size_t lds, hipStream_t stream)
{
    switch (slots) {
    IPTQ_ROWSDYN_CASE(1, 1)
    IPTQ_ROWSDYN_CASE(1, 2)
    IPTQ_ROWSDYN_CASE(1, 3)
    IPTQ_ROWSDYN_CASE(1, 4)
    IPTQ_ROWSDYN_CASE(1, 5)
    IPTQ_ROWSDYN_CASE(1, 6)
    IPTQ_ROWSDYN_CASE(1, 7)
    IPTQ_ROWSDYN_CASE(1, 8)
    default: return false;
    }
}
}  // namespace iptq
