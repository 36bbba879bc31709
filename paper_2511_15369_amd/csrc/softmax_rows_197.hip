// Instantiations of the fixed-row-length softmax for 197 columns (ViT / DeiT at 224x224: 4 lanes per row, 16 rows per wavefront).
#include "softmax_rows.h"

namespace iptq {
IPTQ_DEFINE_ROWS_LAUNCHER(197, 4)
}
