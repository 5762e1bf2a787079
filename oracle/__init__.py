"""fp64 CPU oracle (test infrastructure only).  See flashrnn_oracle.c for what it computes."""
from .oracle import (CELL_LSTM, CELL_GRU, CELL_SLSTM, CELL_ELMAN, CELL_GRU4, build, num_states, num_gates, num_threads, fwd, bwd)  # noqa: F401
