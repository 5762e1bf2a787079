"""Thin ctypes binding over libflashrnn.so (the C ABI of include/flashrnn.h), same entry-point names.

Argument marshalling only: torch supplies device memory and the current HIP stream, every step of
the computation runs inside the library's kernels.  There is no fallback: if the library has not
been built (python -m paper_2412_07752_amd.build) every call raises.
"""
import ctypes
import os

import torch

FLASHRNN_LSTM, FLASHRNN_GRU, FLASHRNN_SLSTM, FLASHRNN_ELMAN, FLASHRNN_GRU4 = 0, 1, 2, 3, 4
FLASHRNN_F32, FLASHRNN_BF16 = 0, 1
FLASHRNN_OK = 0
FLASHRNN_ERR_NULL, FLASHRNN_ERR_SHAPE, FLASHRNN_ERR_UNSUPPORTED = -1, -2, -3
FLASHRNN_ERR_WORKSPACE, FLASHRNN_ERR_LAUNCH, FLASHRNN_ERR_TIMEOUT, FLASHRNN_ERR_SCRATCH = -4, -5, -6, -7
FLASHRNN_STATIC_SCRATCH_BYTES = 16 << 20
STATIC_SCRATCH = "static"   # stands for FLASHRNN_STATIC_SCRATCH in flashrnn_check

# FLASHRNN_LIB=trace selects the library built with per-phase clock stamps (python -m paper_2412_07752_amd.build --trace)
_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)),
                         "libflashrnn_trace.so" if os.environ.get("FLASHRNN_LIB") == "trace" else "libflashrnn.so")
_lib = None


class flashrnn_desc_t(ctypes.Structure):
    _fields_ = [("cell", ctypes.c_int), ("T", ctypes.c_int), ("B", ctypes.c_int), ("NH", ctypes.c_int), ("D", ctypes.c_int),
                ("io_dtype", ctypes.c_int), ("recurrent_grad_clip", ctypes.c_float)]


class FlashRNNError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


def library_path():
    return _LIB_PATH


def lib():
    """The loaded C-ABI library; raises if it was not built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(f"{_LIB_PATH} is missing: build it with `python -m paper_2412_07752_amd.build` "
                               "(there is no CPU fallback)")
        L = ctypes.CDLL(_LIB_PATH)
        dp = ctypes.POINTER(flashrnn_desc_t)
        vp = ctypes.c_void_p
        L.flashrnn_num_states.argtypes = [ctypes.c_int]
        L.flashrnn_num_states.restype = ctypes.c_int
        L.flashrnn_num_gates.argtypes = [ctypes.c_int]
        L.flashrnn_num_gates.restype = ctypes.c_int
        L.flashrnn_gate_cache_bytes.argtypes = [dp]
        L.flashrnn_gate_cache_bytes.restype = ctypes.c_size_t
        L.flashrnn_workspace_bytes.argtypes = [dp]
        L.flashrnn_workspace_bytes.restype = ctypes.c_size_t
        L.flashrnn_fwd.argtypes = [dp] + [vp] * 8
        L.flashrnn_fwd.restype = ctypes.c_int
        L.flashrnn_fwd_static_scratch.argtypes = [dp] + [vp] * 7
        L.flashrnn_fwd_static_scratch.restype = ctypes.c_int
        L.flashrnn_bwd.argtypes = [dp] + [vp] * 12
        L.flashrnn_bwd.restype = ctypes.c_int
        L.flashrnn_bwd_recompute.argtypes = [dp] + [vp] * 12
        L.flashrnn_bwd_recompute.restype = ctypes.c_int
        L.flashrnn_recompute_workspace_bytes.argtypes = [dp]
        L.flashrnn_recompute_workspace_bytes.restype = ctypes.c_size_t
        L.flashrnn_check.argtypes = [dp, vp, vp]
        L.flashrnn_check.restype = ctypes.c_int
        L.flashrnn_plan.argtypes = [dp, ctypes.c_int] + [ctypes.POINTER(ctypes.c_int)] * 3
        L.flashrnn_plan.restype = ctypes.c_int
        L.flashrnn_plan_kernel.argtypes = [dp, ctypes.c_int] + [ctypes.POINTER(ctypes.c_int)] * 3
        L.flashrnn_plan_kernel.restype = ctypes.c_int
        L.flashrnn_profile_enable.argtypes = [ctypes.c_int]
        L.flashrnn_profile_enable.restype = ctypes.c_int
        L.flashrnn_profile_kernel_ms.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_int)]
        L.flashrnn_profile_kernel_ms.restype = ctypes.c_int
        L.flashrnn_trace_phases.argtypes = [dp, vp, ctypes.c_int, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int), vp]
        L.flashrnn_trace_phases.restype = ctypes.c_int
        L.flashrnn_status_string.argtypes = [ctypes.c_int]
        L.flashrnn_status_string.restype = ctypes.c_char_p
        _lib = L
    return _lib


EXPORTS = ["flashrnn_num_states", "flashrnn_num_gates", "flashrnn_gate_cache_bytes", "flashrnn_workspace_bytes", "flashrnn_fwd",
           "flashrnn_fwd_static_scratch", "flashrnn_bwd", "flashrnn_bwd_recompute", "flashrnn_recompute_workspace_bytes", "flashrnn_check", "flashrnn_plan", "flashrnn_plan_kernel", "flashrnn_profile_enable", "flashrnn_profile_kernel_ms",
           "flashrnn_trace_phases", "flashrnn_status_string"]


def status_string(status):
    return lib().flashrnn_status_string(int(status)).decode()


def flashrnn_num_states(cell):
    return lib().flashrnn_num_states(int(cell))


def flashrnn_num_gates(cell):
    return lib().flashrnn_num_gates(int(cell))


def make_desc(cell, T, B, NH, D, io_dtype, recurrent_grad_clip=0.0):
    """recurrent_grad_clip: 0 = off, c > 0 clips R^T dg_t to [-c, c] per step, negative cuts it (backward only)."""
    return flashrnn_desc_t(int(cell), int(T), int(B), int(NH), int(D), int(io_dtype), float(recurrent_grad_clip))


def flashrnn_gate_cache_bytes(desc):
    return lib().flashrnn_gate_cache_bytes(ctypes.byref(desc))


def flashrnn_workspace_bytes(desc):
    return lib().flashrnn_workspace_bytes(ctypes.byref(desc))


def flashrnn_plan(desc, backward=False):
    """(workgroups, CUs per head, waves per workgroup) of the launch the library would use.
    backward: False / 0 the forward call that saves its values, True / 1 the backward call, 2 the forward call that saves nothing."""
    a, b, c = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
    rc = lib().flashrnn_plan(ctypes.byref(desc), int(backward), ctypes.byref(a), ctypes.byref(b), ctypes.byref(c))
    if rc != FLASHRNN_OK:
        raise FlashRNNError(rc, "flashrnn_plan")
    return a.value, b.value, c.value


def flashrnn_plan_kernel(desc, backward=False):
    """(staged: 0 / 1 / 2 = staged with the deep fetch, batch tile rows, workgroups per group) of the kernel that plan uses."""
    a, b, c = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
    rc = lib().flashrnn_plan_kernel(ctypes.byref(desc), int(backward), ctypes.byref(a), ctypes.byref(b), ctypes.byref(c))
    if rc != FLASHRNN_OK:
        raise FlashRNNError(rc, "flashrnn_plan_kernel")
    return a.value, b.value, c.value


def flashrnn_profile_enable(on):
    """on: False / 0 = off, True / 1 = every call, n = every n-th call of each direction carries the two events."""
    rc = lib().flashrnn_profile_enable(int(on))
    if rc != FLASHRNN_OK:
        raise FlashRNNError(rc, "flashrnn_profile_enable")


def flashrnn_profile_kernel_ms(backward):
    """(mean ms, launches) of the persistent kernel of the recorded forward / backward calls."""
    ms, n = ctypes.c_float(), ctypes.c_int()
    rc = lib().flashrnn_profile_kernel_ms(int(bool(backward)), ctypes.byref(ms), ctypes.byref(n))
    if rc != FLASHRNN_OK:
        raise FlashRNNError(rc, "flashrnn_profile_kernel_ms")
    return ms.value, n.value


def flashrnn_trace_phases(desc, workspace, backward, stream=None):
    """(clocks per phase [8], waves recorded) of the last forward / backward call on `workspace`; trace builds only."""
    arr = (ctypes.c_double * 8)()
    n = ctypes.c_int()
    rc = lib().flashrnn_trace_phases(ctypes.byref(desc), _ptr(workspace), int(bool(backward)), arr, ctypes.byref(n), _stream(stream))
    if rc != FLASHRNN_OK:
        raise FlashRNNError(rc, "flashrnn_trace_phases")
    return list(arr), n.value


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _io_dtype(t):
    if t.dtype == torch.bfloat16:
        return FLASHRNN_BF16
    if t.dtype == torch.float32:
        return FLASHRNN_F32
    raise TypeError(f"I/O tensors must be bfloat16 or float32, got {t.dtype}")


def _chk(t, shape, dtype, name, optional=False):
    if t is None:
        if optional:
            return
        raise ValueError(f"{name} is required")
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous device tensor")
    if tuple(t.shape) != tuple(shape) or t.dtype != dtype:
        raise ValueError(f"{name}: got {tuple(t.shape)} {t.dtype}, expected {tuple(shape)} {dtype}")


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def alloc_workspace(desc, device):
    n = flashrnn_workspace_bytes(desc)
    if n == 0:
        raise FlashRNNError(FLASHRNN_ERR_UNSUPPORTED, "flashrnn_workspace_bytes")
    # zero-filled once: a backward call on a workspace that no forward call has used must find clean error words
    return torch.zeros(n, dtype=torch.uint8, device=device)


def flashrnn_fwd_static_scratch(cell, Wx, R, b, states0=None, save_for_backward=True, stream=None, states=None, gate_cache=None):
    """flashrnn_fwd without a workspace: the library works in its own static device array (no allocation in the call
    when `states` and `gate_cache` are passed in).  Returns (states, gate_cache or None)."""
    T, B, G, NH, D = Wx.shape
    S = flashrnn_num_states(cell)
    if G != flashrnn_num_gates(cell):
        raise ValueError("gate axis of Wx does not match the cell")
    dt = Wx.dtype
    desc = make_desc(cell, T, B, NH, D, _io_dtype(Wx))
    _chk(Wx, (T, B, G, NH, D), dt, "Wx")
    _chk(R, (NH, D, G, D), dt, "R")
    _chk(b, (NH, G, D), dt, "b")
    _chk(states0, (S, B, NH, D), torch.float32, "states0", optional=True)
    if states is None:
        states = torch.empty((T + 1, S, B, NH, D), dtype=torch.float32, device=Wx.device)
    _chk(states, (T + 1, S, B, NH, D), torch.float32, "states")
    if save_for_backward and gate_cache is None:
        gate_cache = torch.empty(max(flashrnn_gate_cache_bytes(desc), 16), dtype=torch.uint8, device=Wx.device)
    rc = lib().flashrnn_fwd_static_scratch(ctypes.byref(desc), _ptr(Wx), _ptr(R), _ptr(b), _ptr(states0), _ptr(states),
                                           _ptr(gate_cache) if save_for_backward else None, _stream(stream))
    if rc != FLASHRNN_OK:
        raise FlashRNNError(rc, "flashrnn_fwd_static_scratch")
    return states, (gate_cache if save_for_backward else None)


def flashrnn_fwd(cell, Wx, R, b, states0=None, save_for_backward=True, workspace=None, stream=None, states=None, gate_cache=None):
    """Forward pass.  Wx[T,B,G,NH,D], R[NH,D,G,D], b[NH,G,D] (bf16 or f32), states0[S,B,NH,D] f32 or None.
    Returns (states[T+1,S,B,NH,D] f32, gate_cache or None, workspace)."""
    T, B, G, NH, D = Wx.shape
    S = flashrnn_num_states(cell)
    if G != flashrnn_num_gates(cell):
        raise ValueError("gate axis of Wx does not match the cell")
    dt = Wx.dtype
    desc = make_desc(cell, T, B, NH, D, _io_dtype(Wx))
    _chk(Wx, (T, B, G, NH, D), dt, "Wx")
    _chk(R, (NH, D, G, D), dt, "R")
    _chk(b, (NH, G, D), dt, "b")
    _chk(states0, (S, B, NH, D), torch.float32, "states0", optional=True)
    dev = Wx.device
    if states is None:
        states = torch.empty((T + 1, S, B, NH, D), dtype=torch.float32, device=dev)
    _chk(states, (T + 1, S, B, NH, D), torch.float32, "states")
    if save_for_backward and gate_cache is None:
        gate_cache = torch.empty(max(flashrnn_gate_cache_bytes(desc), 16), dtype=torch.uint8, device=dev)
    if workspace is None:
        workspace = alloc_workspace(desc, dev)
    rc = lib().flashrnn_fwd(ctypes.byref(desc), _ptr(Wx), _ptr(R), _ptr(b), _ptr(states0), _ptr(states),
                            _ptr(gate_cache) if save_for_backward else None, _ptr(workspace), _stream(stream))
    if rc != FLASHRNN_OK:
        raise FlashRNNError(rc, "flashrnn_fwd")
    return states, (gate_cache if save_for_backward else None), workspace


def flashrnn_bwd(cell, R, b, states, gate_cache, dH, dstates_last=None, workspace=None, stream=None, out=None,
                 recurrent_grad_clip=0.0):
    """BPTT.  dH[T,B,NH,D] (I/O dtype).  Returns (dWx[T,B,G,NH,D], dR[NH,D,G,D] f32, db[NH,G,D] f32,
    dstates0[S,B,NH,D] f32).  `out` may pass preallocated (dWx, dR, db, dstates0).  recurrent_grad_clip as in
    flashrnn_desc_t: 0 off, c > 0 clips R^T dg_t to [-c, c] per step, negative cuts it."""
    T, B, NH, D = dH.shape
    S, G = flashrnn_num_states(cell), flashrnn_num_gates(cell)
    dt = dH.dtype
    desc = make_desc(cell, T, B, NH, D, _io_dtype(dH), recurrent_grad_clip)
    _chk(R, (NH, D, G, D), dt, "R")
    _chk(b, (NH, G, D), dt, "b")
    _chk(states, (T + 1, S, B, NH, D), torch.float32, "states")
    _chk(dstates_last, (S, B, NH, D), torch.float32, "dstates_last", optional=True)
    if gate_cache is None or gate_cache.numel() * gate_cache.element_size() < flashrnn_gate_cache_bytes(desc):
        raise ValueError("gate_cache missing or too small")
    dev = dH.device
    if out is None:
        dWx = torch.empty((T, B, G, NH, D), dtype=dt, device=dev)
        dR = torch.empty((NH, D, G, D), dtype=torch.float32, device=dev)
        db = torch.empty((NH, G, D), dtype=torch.float32, device=dev)
        ds0 = torch.empty((S, B, NH, D), dtype=torch.float32, device=dev)
    else:
        dWx, dR, db, ds0 = out
    if workspace is None:
        workspace = alloc_workspace(desc, dev)
    rc = lib().flashrnn_bwd(ctypes.byref(desc), _ptr(R), _ptr(b), _ptr(states), _ptr(gate_cache), _ptr(dH), _ptr(dstates_last),
                            _ptr(dWx), _ptr(dR), _ptr(db), _ptr(ds0), _ptr(workspace), _stream(stream))
    if rc != FLASHRNN_OK:
        raise FlashRNNError(rc, "flashrnn_bwd")
    return dWx, dR, db, ds0


def flashrnn_bwd_recompute(cell, Wx, R, b, states, dH, dstates_last=None, workspace=None, stream=None, out=None, recurrent_grad_clip=0.0):
    """BPTT without saved values: they are formed again from Wx, R, b and the states, window by window.  Arguments and
    results as flashrnn_bwd, with Wx[T,B,G,NH,D] in place of the gate cache; `workspace` needs
    flashrnn_recompute_workspace_bytes() bytes."""
    T, B, NH, D = dH.shape
    S, G = flashrnn_num_states(cell), flashrnn_num_gates(cell)
    dt = dH.dtype
    desc = make_desc(cell, T, B, NH, D, _io_dtype(dH), recurrent_grad_clip)
    _chk(Wx, (T, B, G, NH, D), dt, "Wx")
    _chk(R, (NH, D, G, D), dt, "R")
    _chk(b, (NH, G, D), dt, "b")
    _chk(states, (T + 1, S, B, NH, D), torch.float32, "states")
    _chk(dstates_last, (S, B, NH, D), torch.float32, "dstates_last", optional=True)
    dev = dH.device
    if out is None:
        out = (torch.empty((T, B, G, NH, D), dtype=dt, device=dev), torch.empty((NH, D, G, D), dtype=torch.float32, device=dev),
               torch.empty((NH, G, D), dtype=torch.float32, device=dev), torch.empty((S, B, NH, D), dtype=torch.float32, device=dev))
    dWx, dR, db, ds0 = out
    if workspace is None:
        n = lib().flashrnn_recompute_workspace_bytes(ctypes.byref(desc))
        if n == 0:
            raise FlashRNNError(FLASHRNN_ERR_UNSUPPORTED, "flashrnn_recompute_workspace_bytes")
        workspace = torch.zeros(n, dtype=torch.uint8, device=dev)
    rc = lib().flashrnn_bwd_recompute(ctypes.byref(desc), _ptr(Wx), _ptr(R), _ptr(b), _ptr(states), _ptr(dH), _ptr(dstates_last),
                                      _ptr(dWx), _ptr(dR), _ptr(db), _ptr(ds0), _ptr(workspace), _stream(stream))
    if rc != FLASHRNN_OK:
        raise FlashRNNError(rc, "flashrnn_bwd_recompute")
    return dWx, dR, db, ds0, workspace


def flashrnn_check(desc, workspace, stream=None):
    """Synchronizes and raises FlashRNNError if a kernel of the last call reported a timeout."""
    ws = ctypes.c_void_p(1) if isinstance(workspace, str) and workspace == STATIC_SCRATCH else _ptr(workspace)
    rc = lib().flashrnn_check(ctypes.byref(desc), ws, _stream(stream))
    if rc != FLASHRNN_OK:
        raise FlashRNNError(rc, "flashrnn_check")
