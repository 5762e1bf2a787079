"""MI355X-native FlashRNN time-step loop (LSTM / GRU / sLSTM, forward and BPTT backward).

The compute path is the C-ABI library built from csrc/ (HIP for gfx950); `api` is a thin ctypes
binding over it and `synth` draws the seeded synthetic workloads.  Nothing here falls back to a CPU
implementation: calls raise if the HIP library has not been built.
"""
from . import synth  # noqa: F401
