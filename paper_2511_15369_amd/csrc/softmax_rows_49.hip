// Instantiations of the fixed-row-length softmax for 49 columns (Swin 7x7 windows: 2 lanes per row, 32 rows per wavefront).
#include "softmax_rows.h"

namespace iptq {
IPTQ_DEFINE_ROWS_LAUNCHER(49, 2)
}
