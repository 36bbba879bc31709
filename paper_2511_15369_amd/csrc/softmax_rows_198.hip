// Instantiations of the fixed-row-length softmax for 198 columns (DeiT with a distillation token: 4 lanes per row, 16 rows per wavefront).
#include "softmax_rows.h"

namespace iptq {
IPTQ_DEFINE_ROWS_LAUNCHER(198, 4)
}
