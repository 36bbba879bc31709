// One-workgroup-per-row softmax kernel, 8 wavefronts per row, 11 to 13 passes.
#include "softmax_wgrow.h"

namespace iptq {
bool wgrow_launch_w8_hi(const WideArgs &A, int passes, int mode, dim3 grid, hipStream_t stream)
{
    switch (passes) {
    IPTQ_WGROW_CASE(8, 11)
    IPTQ_WGROW_CASE(8, 12)
    IPTQ_WGROW_CASE(8, 13)
    default: return false;
    }
}
}  // namespace iptq
