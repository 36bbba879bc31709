// 198 columns with 8 lanes per row (8 rows per wavefront), used for short launches.
#include "softmax_rows.h"

namespace iptq {
IPTQ_DEFINE_ROWS_LAUNCHER(198, 8)
}
