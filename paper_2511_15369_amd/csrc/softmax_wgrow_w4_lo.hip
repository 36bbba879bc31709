// One-workgroup-per-row softmax kernel, 4 wavefronts per row, 5 to 9 passes.
#include "softmax_wgrow.h"

namespace iptq {
bool wgrow_launch_w4_lo(const WideArgs &A, int passes, int mode, dim3 grid, hipStream_t stream)
{
    switch (passes) {
    IPTQ_WGROW_CASE(4, 5)
    IPTQ_WGROW_CASE(4, 6)
    IPTQ_WGROW_CASE(4, 7)
    IPTQ_WGROW_CASE(4, 8)
    IPTQ_WGROW_CASE(4, 9)
    default: return false;
    }
}
}  // namespace iptq
