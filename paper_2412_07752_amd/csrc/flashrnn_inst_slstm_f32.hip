// Persistent-kernel instantiations: slstm, f32 I/O.
#define FRNN_CELL flashrnn::CELL_SLSTM
#define FRNN_G 4
#define FRNN_BF16 0
#include "flashrnn_inst.h"

namespace flashrnn {
KernelTable table_slstm_f32() { return make_table(); }
}  // namespace flashrnn
