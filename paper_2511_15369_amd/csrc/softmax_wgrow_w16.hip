// One-workgroup-per-row softmax kernel, 16 wavefronts per row, 7 to 10 passes.
#include "softmax_wgrow.h"

namespace iptq {
bool wgrow_launch_w16(const WideArgs &A, int passes, int mode, dim3 grid, hipStream_t stream)
{
    switch (passes) {
    IPTQ_WGROW_CASE(16, 7)
    IPTQ_WGROW_CASE(16, 8)
    IPTQ_WGROW_CASE(16, 9)
    IPTQ_WGROW_CASE(16, 10)
    default: return false;
    }
}
}  // namespace iptq
