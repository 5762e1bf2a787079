"""The entry point that allocates nothing: flashrnn_fwd_static_scratch works in the library's static device array
instead of a caller's workspace.  Same kernels as flashrnn_fwd, so the outputs must agree bit for bit (and with the
oracle within the usual tolerance).  Two calls in a row, the second one smaller: the array keeps the first call's
content, and everything the second call needs cleared (exchange stamps, error words) it must clear itself."""
import ctypes

import numpy as np
import pytest
import torch

import parity_util as pu
from paper_2412_07752_amd import api, synth
from paper_2412_07752_amd.synth import CELL_LSTM, CELL_SLSTM, Workload

pytestmark = pytest.mark.gpu


def _both(w):
    inp = synth.make_inputs(w)
    Wx, R, b = (pu.to_device(inp[k], w.dtype) for k in ("Wx", "R", "b"))
    s0 = pu.to_device(inp["states0"], "f32")
    desc = api.make_desc(w.cell, w.T, w.B, w.NH, w.D, api.FLASHRNN_BF16 if w.dtype == "bf16" else api.FLASHRNN_F32)
    # outputs are allocated before the call under test: the call itself goes straight through the C ABI
    states = torch.full((w.T + 1, w.S, w.B, w.NH, w.D), float("nan"), dtype=torch.float32, device="cuda")
    cache = torch.zeros(api.flashrnn_gate_cache_bytes(desc), dtype=torch.uint8, device="cuda")
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    print(f"static-scratch call: {w.name}", flush=True)
    rc = api.lib().flashrnn_fwd_static_scratch(ctypes.byref(desc), Wx.data_ptr(), R.data_ptr(), b.data_ptr(),
                                               None if s0 is None else s0.data_ptr(), states.data_ptr(), cache.data_ptr(), stream)
    assert rc == api.FLASHRNN_OK, api.status_string(rc)
    api.flashrnn_check(desc, api.STATIC_SCRATCH)
    ref_states, ref_cache, ws = api.flashrnn_fwd(w.cell, Wx, R, b, s0)
    api.flashrnn_check(desc, ws)
    torch.cuda.synchronize()
    assert torch.equal(states, ref_states), f"{w.name}: states differ from flashrnn_fwd's"
    assert torch.equal(cache, ref_cache[:cache.numel()]), f"{w.name}: saved values differ from flashrnn_fwd's"
    oracle_out = pu.run_oracle(w, inp)
    gpu = {"states": pu.to_host64(states)}
    pu.assert_close(w, pu.compare(w, gpu, oracle_out))
    pu.assert_states_elementwise(w, gpu, oracle_out)


def test_two_calls_in_a_row_second_one_smaller():
    # a head split over four workgroups (exchange buffers and error words live in the static array), 13 ragged rows
    big = Workload("static_big", CELL_SLSTM, 14, 13, 2, 256, "bf16", False, bias="forget3", init="uniform0.1", seed=11)
    d = api.make_desc(big.cell, big.T, big.B, big.NH, big.D, api.FLASHRNN_BF16)
    assert api.flashrnn_plan_kernel(d)[2] > 1
    _both(big)
    # smaller in every direction, same kind of plan: it must not see the first call's stamps or packed weights
    small = Workload("static_small", CELL_SLSTM, 5, 3, 1, 208, "bf16", False, bias="forget3", init="uniform0.1", seed=12)
    _both(small)
    # and a one-workgroup plan in the other dtype
    _both(Workload("static_f32", CELL_LSTM, 6, 4, 2, 32, "f32", False, bias="uniform0.1", seed=13))


def test_too_large_for_the_static_array_is_refused():
    """One head of 1024 units needs an 8 MiB packed copy of R per gate set (4 gates x 1024 x 1024 bf16) plus exchange buffers."""
    T, B, NH, D = 2, 2, 3, 1024
    desc = api.make_desc(CELL_LSTM, T, B, NH, D, api.FLASHRNN_BF16)
    assert NH * 4 * D * D * 2 > api.FLASHRNN_STATIC_SCRATCH_BYTES
    Wx = torch.zeros((T, B, 4, NH, D), dtype=torch.bfloat16, device="cuda")
    R = torch.zeros((NH, D, 4, D), dtype=torch.bfloat16, device="cuda")
    b = torch.zeros((NH, 4, D), dtype=torch.bfloat16, device="cuda")
    states = torch.empty((T + 1, 2, B, NH, D), dtype=torch.float32, device="cuda")
    rc = api.lib().flashrnn_fwd_static_scratch(ctypes.byref(desc), Wx.data_ptr(), R.data_ptr(), b.data_ptr(), None, states.data_ptr(), None, None)
    assert rc == api.FLASHRNN_ERR_SCRATCH
    torch.cuda.synchronize()
