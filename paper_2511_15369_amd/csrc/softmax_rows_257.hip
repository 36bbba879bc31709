// Instantiations of the fixed-row-length softmax for 257 columns (ViT-L/14 at 224x224: 8 lanes per row, 8 rows per wavefront).
#include "softmax_rows.h"

namespace iptq {
IPTQ_DEFINE_ROWS_LAUNCHER(257, 8)
}
