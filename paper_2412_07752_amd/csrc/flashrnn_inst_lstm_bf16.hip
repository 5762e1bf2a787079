// Persistent-kernel instantiations: lstm, bf16 I/O.
#define FRNN_CELL flashrnn::CELL_LSTM
#define FRNN_G 4
#define FRNN_BF16 1
#include "flashrnn_inst.h"

namespace flashrnn {
KernelTable table_lstm_bf16() { return make_table(); }
}  // namespace flashrnn
