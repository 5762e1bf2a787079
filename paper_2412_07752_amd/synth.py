"""Seeded synthetic inputs shaped like the paper's runtime workloads (Sec. 6.1: random tensors,
d = NH x DH, batch 16, T = 256..2048), and the five named benchmark configurations.

This module holds no arithmetic of the method itself: it only draws random tensors with numpy,
rounds them once to the I/O dtype (so the CPU oracle and the GPU path consume identical values) and
names shapes.  It is the only module shared by the oracle-side tests and the GPU-side code.
"""
from dataclasses import dataclass, field

import numpy as np

CELL_LSTM, CELL_GRU, CELL_SLSTM, CELL_ELMAN, CELL_GRU4 = 0, 1, 2, 3, 4
CELL_NAMES = {CELL_LSTM: "lstm", CELL_GRU: "gru", CELL_SLSTM: "slstm", CELL_ELMAN: "elman", CELL_GRU4: "gru4"}
NUM_STATES = {CELL_LSTM: 2, CELL_GRU: 1, CELL_SLSTM: 4, CELL_ELMAN: 1, CELL_GRU4: 1}
NUM_GATES = {CELL_LSTM: 4, CELL_GRU: 3, CELL_SLSTM: 4, CELL_ELMAN: 1, CELL_GRU4: 4}
FORGET_GATE = 1  # index of the forget gate on the G axis (order i, f, z, o)


def round_to_bf16(a):
    """Round float32 values to the nearest bfloat16 (ties to even); result stays float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32)
    rounded = (bits + np.uint32(0x7FFF) + ((bits >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32)


def bf16_bits(a):
    """uint16 bit patterns of float32 values that are already bfloat16-representable."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(u):
    return (np.ascontiguousarray(u, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class Workload:
    name: str
    cell: int
    T: int
    B: int
    NH: int
    D: int
    dtype: str            # "f32" or "bf16": dtype of Wx, R, b, dH, dWx
    backward: bool
    bias: str = "zero"    # "zero" | "forget3" | "uniform0.1" | "forget_linspace_3_6"
    init: str = "zero"    # "zero" | "uniform0.1" | "uniform0.1_bounded" (sLSTM: |c_0| <= n_0, so that |h| <= 1 from the start)
    seed: int = 0
    wx: str = "normal"    # "normal": N(0,1) | "large_mix": N(0,1) plus offsets of 0, +-50, +-100, +-200 (saturated gates)
    extra: dict = field(default_factory=dict)

    @property
    def G(self):
        return NUM_GATES[self.cell]

    @property
    def S(self):
        return NUM_STATES[self.cell]


# The five benchmark configurations (index 0 is the small case the oracle runs in milliseconds,
# index 1 is the one the headline metric is quoted on).
CONFIGS = [
    Workload("C1_lstm_fwd_f32_B4_T32_NH1_D64", CELL_LSTM, 32, 4, 1, 64, "f32", False),
    Workload("C2_slstm_fwdbwd_bf16_B16_T256_NH4_D192", CELL_SLSTM, 256, 16, 4, 192, "bf16", True, bias="forget3"),
    Workload("C3_gru_fwdbwd_bf16_B64_T512_NH8_D128", CELL_GRU, 512, 64, 8, 128, "bf16", True, bias="uniform0.1"),
    Workload("C4_lstm_fwd_bf16_B16_T1024_NH1_D768", CELL_LSTM, 1024, 16, 1, 768, "bf16", False),
    Workload("C5_slstm_fwdbwd_bf16_B32_T2048_NH8_D256", CELL_SLSTM, 2048, 32, 8, 256, "bf16", True,
             bias="forget_linspace_3_6", init="uniform0.1"),
]


def make_inputs(w: Workload):
    """Draw the tensors of one workload.  One sub-stream per tensor (order Wx, R, b, states0, dH),
    all float32, already rounded to the I/O dtype where the I/O dtype is bf16.

    Returns dict with Wx[T,B,G,NH,D], R[NH,D,G,D], b[NH,G,D], states0[S,B,NH,D] or None,
    dH[T,B,NH,D] or None.
    """
    T, B, NH, D, G, S = w.T, w.B, w.NH, w.D, w.G, w.S
    rnd = round_to_bf16 if w.dtype == "bf16" else (lambda a: np.ascontiguousarray(a, dtype=np.float32))

    def stream(k):
        return np.random.default_rng([w.seed, k])

    out = {}
    Wx = stream(0).standard_normal((T, B, G, NH, D), dtype=np.float32)
    if w.wx == "large_mix":
        # the regime the sLSTM stabilizer exists for: about a third of the pre-activations far out in either tail
        levels = np.array([0.0, 0.0, 0.0, 0.0, 50.0, -50.0, 100.0, -100.0, 200.0, -200.0], dtype=np.float32)
        off = levels[stream(5).integers(0, len(levels), size=Wx.shape)]
        if w.cell == CELL_SLSTM and w.init == "zero":
            # an empty cell (n_0 = 0, m_0 = 0) cannot hold exp(i - m) below the float32 range as its normalizer:
            # the first input gate stays on the non-negative side
            off[0, :, 0] = np.abs(off[0, :, 0])
        Wx = Wx + off
    elif w.wx != "normal":
        raise ValueError(w.wx)
    out["Wx"] = rnd(Wx)
    out["R"] = rnd(stream(1).standard_normal((NH, D, G, D), dtype=np.float32) * np.float32(D ** -0.5))
    b = np.zeros((NH, G, D), dtype=np.float32)
    if w.bias == "forget3":
        b[:, FORGET_GATE, :] = 3.0
    elif w.bias == "uniform0.1":
        b = stream(2).uniform(-0.1, 0.1, size=(NH, G, D)).astype(np.float32)
    elif w.bias == "forget_linspace_3_6":
        b[:, FORGET_GATE, :] = np.linspace(3.0, 6.0, NH, dtype=np.float32)[:, None]
    elif w.bias != "zero":
        raise ValueError(w.bias)
    out["b"] = rnd(b)
    if w.init in ("uniform0.1", "uniform0.1_bounded"):
        s0 = stream(3).uniform(0.0, 0.1, size=(S, B, NH, D)).astype(np.float32)
        if w.cell == CELL_SLSTM:
            s0[3] = 0.0  # stabilizer starts at zero
            if w.init == "uniform0.1_bounded":
                s0[1] *= s0[2] * np.float32(10.0)   # c_0 in [0, n_0]: the cell keeps |c_t| <= n_t, hence |h_t| <= 1
        out["states0"] = s0  # states are float32 in every configuration
    elif w.init == "zero":
        out["states0"] = None
    else:
        raise ValueError(w.init)
    out["dH"] = rnd(stream(4).standard_normal((T, B, NH, D), dtype=np.float32)) if w.backward else None
    return out
