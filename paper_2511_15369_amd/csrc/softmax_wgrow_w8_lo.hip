// One-workgroup-per-row softmax kernel, 8 wavefronts per row, 7 to 10 passes.
#include "softmax_wgrow.h"

namespace iptq {
bool wgrow_launch_w8_lo(const WideArgs &A, int passes, int mode, dim3 grid, hipStream_t stream)
{
    switch (passes) {
    IPTQ_WGROW_CASE(8, 7)
    IPTQ_WGROW_CASE(8, 8)
    IPTQ_WGROW_CASE(8, 9)
    IPTQ_WGROW_CASE(8, 10)
    default: return false;
    }
}
}  // namespace iptq
