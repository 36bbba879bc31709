// Run-time-row-length softmax slab kernel, 2 lanes per row.
#include "softmax_rowsdyn.h"

namespace iptq {
IPTQ_DEFINE_ROWSDYN_LAUNCHER(2)
}
