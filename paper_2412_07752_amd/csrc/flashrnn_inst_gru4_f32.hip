// Persistent-kernel instantiations: gru4 (the GRU as App. A prints it), f32 I/O.
#define FRNN_CELL flashrnn::CELL_GRU4
#define FRNN_G 4
#define FRNN_BF16 0
#include "flashrnn_inst.h"

namespace flashrnn {
KernelTable table_gru4_f32() { return make_table(); }
}  // namespace flashrnn
