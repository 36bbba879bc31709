// One-wavefront-per-row softmax kernel, 1 to 6 passes of 64 blocks.
#include "softmax_wide.h"

namespace iptq {
bool wide_launch_p1_6(const WideArgs &A, int passes, int mode, dim3 grid, hipStream_t stream)
{
    switch (passes) {
    IPTQ_WIDE_CASE(1)
    IPTQ_WIDE_CASE(2)
    IPTQ_WIDE_CASE(3)
    IPTQ_WIDE_CASE(4)
    IPTQ_WIDE_CASE(5)
    IPTQ_WIDE_CASE(6)
    default: return false;
    }
}
}  // namespace iptq
