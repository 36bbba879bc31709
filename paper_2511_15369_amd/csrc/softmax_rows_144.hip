// Instantiations of the fixed-row-length softmax for 144 columns (Swin 12x12 windows: 4 lanes per row, 16 rows per wavefront).
#include "softmax_rows.h"

namespace iptq {
IPTQ_DEFINE_ROWS_LAUNCHER(144, 4)
}
