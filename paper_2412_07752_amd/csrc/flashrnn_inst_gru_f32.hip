// Persistent-kernel instantiations: gru, f32 I/O.
#define FRNN_CELL flashrnn::CELL_GRU
#define FRNN_G 3
#define FRNN_BF16 0
#include "flashrnn_inst.h"

namespace flashrnn {
KernelTable table_gru_f32() { return make_table(); }
}  // namespace flashrnn
