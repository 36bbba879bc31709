// One-wavefront-per-row softmax kernel, 14 to 16 passes of 64 blocks.
#include "softmax_wide.h"

namespace iptq {
bool wide_launch_p14_16(const WideArgs &A, int passes, int mode, dim3 grid, hipStream_t stream)
{
    switch (passes) {
    IPTQ_WIDE_CASE(14)
    IPTQ_WIDE_CASE(15)
    IPTQ_WIDE_CASE(16)
    default: return false;
    }
}
}  // namespace iptq
