// Run-time-row-length softmax slab kernel, 8 lanes per row, 5 to 8 blocks per lane.
#include "softmax_rowsdyn.h"

namespace iptq {
bool rowsdyn_launch_k8(const DynArgs &A, int slots, int mode, dim3 grid, dim3 block, size_t lds, hipStream_t stream)
{
    switch (slots) {
    IPTQ_ROWSDYN_CASE(8, 5)
    IPTQ_ROWSDYN_CASE(8, 6)
    IPTQ_ROWSDYN_CASE(8, 7)
    IPTQ_ROWSDYN_CASE(8, 8)
    default: return false;
    }
}
}  // namespace iptq
