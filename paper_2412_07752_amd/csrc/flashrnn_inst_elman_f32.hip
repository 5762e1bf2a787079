// Persistent-kernel instantiations: elman, f32 I/O.
#define FRNN_CELL flashrnn::CELL_ELMAN
#define FRNN_G 1
#define FRNN_BF16 0
#include "flashrnn_inst.h"

namespace flashrnn {
KernelTable table_elman_f32() { return make_table(); }
}  // namespace flashrnn
