// Persistent-kernel instantiations: elman, bf16 I/O.
#define FRNN_CELL flashrnn::CELL_ELMAN
#define FRNN_G 1
#define FRNN_BF16 1
#include "flashrnn_inst.h"

namespace flashrnn {
KernelTable table_elman_bf16() { return make_table(); }
}  // namespace flashrnn
