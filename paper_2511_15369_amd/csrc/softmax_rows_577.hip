// Instantiations of the fixed-row-length softmax for 577 columns (ViT at 384x384 / 16: 16 lanes per row, 4 rows per wavefront).
#include "softmax_rows.h"

namespace iptq {
IPTQ_DEFINE_ROWS_LAUNCHER(577, 16)
}
