// One-wavefront-per-row softmax kernel, 11 to 13 passes of 64 blocks.
#include "softmax_wide.h"

namespace iptq {
bool wide_launch_p11_13(const WideArgs &A, int passes, int mode, dim3 grid, hipStream_t stream)
{
    switch (passes) {
    IPTQ_WIDE_CASE(11)
    IPTQ_WIDE_CASE(12)
    IPTQ_WIDE_CASE(13)
    default: return false;
    }
}
}  // namespace iptq
