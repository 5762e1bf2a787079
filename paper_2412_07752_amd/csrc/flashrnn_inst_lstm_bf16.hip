// Persistent-kernel instantiations: lstm, bf16 I/O.
#define FRNN_CELL flashrnn::CELL_LSTM
#define FRNN_G 4
#define FRNN_BF16 1
#include "flashrnn_inst.h"

namespace flashrnn {
KernelTable table_lstm_bf16() { return KernelTable{kEntries, (int)(sizeof(kEntries) / sizeof(kEntries[0]))}; }
}  // namespace flashrnn
