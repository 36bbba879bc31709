// Run-time-row-length softmax slab kernel, 16 lanes per row, up to 8 blocks per lane.
#include "softmax_rowsdyn.h"

namespace iptq {
IPTQ_DEFINE_ROWSDYN_LAUNCHER(16)
}
