// Persistent-kernel instantiations: gru4 (the GRU as App. A prints it), bf16 I/O.
#define FRNN_CELL flashrnn::CELL_GRU4
#define FRNN_G 4
#define FRNN_BF16 1
#include "flashrnn_inst.h"

namespace flashrnn {
KernelTable table_gru4_bf16() { return make_table(); }
}  // namespace flashrnn
