// Run-time-row-length softmax slab kernel, 16 lanes per row, 9 or 10 blocks per lane.
#include "softmax_rowsdyn.h"

namespace iptq {
bool rowsdyn_launch_k16_long(const DynArgs &A, int slots, int mode, dim3 grid, dim3 block, size_t lds, hipStream_t stream)
{
    switch (slots) {
    IPTQ_ROWSDYN_CASE(16, 9)
    IPTQ_ROWSDYN_CASE(16, 10)
    default: return false;
    }
}
}  // namespace iptq
