// One-wavefront-per-row softmax kernel, 7 to 10 passes of 64 blocks.
#include "softmax_wide.h"

namespace iptq {
bool wide_launch_p7_10(const WideArgs &A, int passes, int mode, dim3 grid, hipStream_t stream)
{
    switch (passes) {
    IPTQ_WIDE_CASE(7)
    IPTQ_WIDE_CASE(8)
    IPTQ_WIDE_CASE(9)
    IPTQ_WIDE_CASE(10)
    default: return false;
    }
}
}  // namespace iptq
