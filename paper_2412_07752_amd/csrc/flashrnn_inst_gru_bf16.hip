// Persistent-kernel instantiations: gru, bf16 I/O.
#define FRNN_CELL flashrnn::CELL_GRU
#define FRNN_G 3
#define FRNN_BF16 1
#include "flashrnn_inst.h"

namespace flashrnn {
KernelTable table_gru_bf16() { return make_table(); }
}  // namespace flashrnn
