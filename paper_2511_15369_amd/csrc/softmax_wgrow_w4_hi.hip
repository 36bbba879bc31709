// One-workgroup-per-row softmax kernel, 4 wavefronts per row, 10 to 13 passes.
#include "softmax_wgrow.h"

namespace iptq {
bool wgrow_launch_w4_hi(const WideArgs &A, int passes, int mode, dim3 grid, hipStream_t stream)
{
    switch (passes) {
    IPTQ_WGROW_CASE(4, 10)
    IPTQ_WGROW_CASE(4, 11)
    IPTQ_WGROW_CASE(4, 12)
    IPTQ_WGROW_CASE(4, 13)
    default: return false;
    }
}
}  // namespace iptq
