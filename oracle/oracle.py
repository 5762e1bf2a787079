"""ctypes front end of the plain-C fp64 oracle (flashrnn_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by bench.py's
cpu_baseline leg.  The product path (the HIP library and its Python binding) never touches it.

All arrays are C-contiguous numpy float64 in the layouts of the C file:
  Wx[T,B,G,NH,D]  R[NH,D,G,D]  b[NH,G,D]  states[T+1,S,B,NH,D]  dH[T,B,NH,D]
"""
import ctypes
import os
import subprocess

import numpy as np

CELL_LSTM, CELL_GRU, CELL_SLSTM, CELL_ELMAN, CELL_GRU4 = 0, 1, 2, 3, 4

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "flashrnn_oracle.c")
_LIB = os.path.join(_HERE, "libflashrnn_oracle.so")
_lib = None


def build(force=False):
    """Compile the oracle with gcc (plain C, OpenMP over head x batch)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", _SRC, "-o", _LIB, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        lib.oracle_fwd.argtypes = [ctypes.c_int] * 5 + [dp] * 5
        lib.oracle_fwd.restype = ctypes.c_int
        lib.oracle_bwd.argtypes = [ctypes.c_int] * 5 + [dp] * 10
        lib.oracle_bwd.restype = ctypes.c_int
        lib.oracle_bwd_clipped.argtypes = [ctypes.c_int] * 5 + [dp] * 6 + [ctypes.c_double] + [dp] * 4
        lib.oracle_bwd_clipped.restype = ctypes.c_int
        for f in (lib.oracle_num_states, lib.oracle_num_gates):
            f.argtypes = [ctypes.c_int]
            f.restype = ctypes.c_int
        lib.oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_states(cell):
    return _load().oracle_num_states(int(cell))


def num_gates(cell):
    return _load().oracle_num_gates(int(cell))


def num_threads():
    return _load().oracle_num_threads()


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _c(a, shape, name):
    a = np.ascontiguousarray(a, dtype=np.float64)
    if a.shape != tuple(shape):
        raise ValueError(f"{name}: shape {a.shape}, expected {tuple(shape)}")
    return a


def fwd(cell, Wx, R, b, states0=None):
    """Forward pass; returns states[T+1,S,B,NH,D] (slot 0 = initial states)."""
    T, B, G, NH, D = Wx.shape
    S = num_states(cell)
    if G != num_gates(cell):
        raise ValueError("gate axis does not match the cell")
    Wx = _c(Wx, (T, B, G, NH, D), "Wx")
    R = _c(R, (NH, D, G, D), "R")
    b = _c(b, (NH, G, D), "b")
    if states0 is not None:
        states0 = _c(states0, (S, B, NH, D), "states0")
    states = np.empty((T + 1, S, B, NH, D), dtype=np.float64)
    rc = _load().oracle_fwd(int(cell), T, B, NH, D, _p(Wx), _p(R), _p(b), _p(states0), _p(states))
    if rc != 0:
        raise RuntimeError(f"oracle_fwd failed ({rc})")
    return states


def bwd(cell, Wx, R, b, states, dH, dstates_last=None, recurrent_clip=None):
    """BPTT; returns (dWx, dR, db, dstates0).  recurrent_clip (Sec. 4.1): None = off, c >= 0 clips every value of the
    recurrent term R^T dg_t to [-c, c] after each step (0 cuts it)."""
    T, B, G, NH, D = Wx.shape
    S = num_states(cell)
    Wx = _c(Wx, (T, B, G, NH, D), "Wx")
    R = _c(R, (NH, D, G, D), "R")
    b = _c(b, (NH, G, D), "b")
    states = _c(states, (T + 1, S, B, NH, D), "states")
    dH = _c(dH, (T, B, NH, D), "dH")
    if dstates_last is not None:
        dstates_last = _c(dstates_last, (S, B, NH, D), "dstates_last")
    dWx = np.empty_like(Wx)
    dR = np.empty_like(R)
    db = np.empty_like(b)
    ds0 = np.empty((S, B, NH, D), dtype=np.float64)
    clip = -1.0 if recurrent_clip is None else float(recurrent_clip)
    if recurrent_clip is not None and not clip >= 0.0:
        raise ValueError("recurrent_clip must be >= 0 or None")
    rc = _load().oracle_bwd_clipped(int(cell), T, B, NH, D, _p(Wx), _p(R), _p(b), _p(states), _p(dH), _p(dstates_last),
                                    ctypes.c_double(clip), _p(dWx), _p(dR), _p(db), _p(ds0))
    if rc != 0:
        raise RuntimeError(f"oracle_bwd failed ({rc})")
    return dWx, dR, db, ds0
