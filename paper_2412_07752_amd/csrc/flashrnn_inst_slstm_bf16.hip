// Persistent-kernel instantiations: slstm, bf16 I/O.
#define FRNN_CELL flashrnn::CELL_SLSTM
#define FRNN_G 4
#define FRNN_BF16 1
#include "flashrnn_inst.h"

namespace flashrnn {
KernelTable table_slstm_bf16() { return make_table(); }
}  // namespace flashrnn
