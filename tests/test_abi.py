"""CPU-only checks of the boundary: the library loads, exports every symbol the header declares,
and rejects bad descriptors without touching a GPU."""
import ctypes
import os
import re

import pytest

from paper_2412_07752_amd import api

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "flashrnn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(flashrnn_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = api.lib()
    names = _declared_symbols()
    assert set(names) == set(api.EXPORTS), (names, api.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_cell_tables_match_paper_appendix_a():
    assert [api.flashrnn_num_states(c) for c in (0, 1, 2, 3, 4)] == [2, 1, 4, 1, 1]
    assert [api.flashrnn_num_gates(c) for c in (0, 1, 2, 3, 4)] == [4, 3, 4, 1, 4]
    assert api.flashrnn_num_states(7) == -1 and api.flashrnn_num_gates(-1) == -1


def test_status_strings():
    seen = set()
    for s in range(0, -8, -1):
        txt = api.status_string(s)
        assert txt and txt not in seen
        seen.add(txt)
    assert "unknown" in api.status_string(-99)


@pytest.mark.parametrize("bad", [dict(cell=5), dict(T=-1), dict(B=0), dict(NH=0), dict(D=0), dict(io_dtype=3),
                                 dict(recurrent_grad_clip=float("nan"))])
def test_bad_descriptors_are_rejected_on_the_host(bad):
    kw = dict(cell=0, T=4, B=2, NH=1, D=16, io_dtype=api.FLASHRNN_F32)
    kw.update(bad)
    d = api.make_desc(**kw)
    assert api.flashrnn_gate_cache_bytes(d) == 0
    assert api.flashrnn_workspace_bytes(d) == 0
    rc = api.lib().flashrnn_fwd(ctypes.byref(d), None, None, None, None, None, None, None, None)
    assert rc == api.FLASHRNN_ERR_SHAPE
    rc = api.lib().flashrnn_bwd(ctypes.byref(d), *([None] * 12))
    assert rc == api.FLASHRNN_ERR_SHAPE


def test_time_step_slabs_beyond_32_bit_offsets_are_refused():
    """The kernels address one time step of a tensor with 32-bit byte offsets: a shape whose per-step slab reaches 2 GiB
    must be refused, not run with dropped accesses."""
    d = api.make_desc(2, 4, 4096, 64, 1024, api.FLASHRNN_BF16)   # sLSTM states: 4 * 4 B * 2^28 units per step
    assert api.flashrnn_workspace_bytes(d) == 0
    assert api.lib().flashrnn_fwd(ctypes.byref(d), *([None] * 8)) == api.FLASHRNN_ERR_UNSUPPORTED
    d = api.make_desc(2, 4, 64, 64, 1024, api.FLASHRNN_BF16)
    assert api.lib().flashrnn_fwd(ctypes.byref(d), *([None] * 8)) == api.FLASHRNN_ERR_NULL


def test_static_scratch_entry_checks_arguments_first():
    d = api.make_desc(0, 4, 2, 1, 24, api.FLASHRNN_BF16)
    assert api.lib().flashrnn_fwd_static_scratch(ctypes.byref(d), *([None] * 7)) == api.FLASHRNN_ERR_UNSUPPORTED
    assert api.lib().flashrnn_fwd_static_scratch(None, *([None] * 7)) == api.FLASHRNN_ERR_NULL


def test_unsupported_head_size_and_null_pointers():
    d = api.make_desc(0, 4, 2, 1, 24, api.FLASHRNN_BF16)  # D not a multiple of 16
    assert api.lib().flashrnn_fwd(ctypes.byref(d), *([None] * 8)) == api.FLASHRNN_ERR_UNSUPPORTED
    d = api.make_desc(0, 4, 2, 1, 32, api.FLASHRNN_BF16)
    assert api.lib().flashrnn_fwd(ctypes.byref(d), *([None] * 8)) == api.FLASHRNN_ERR_NULL
    assert api.lib().flashrnn_bwd(ctypes.byref(d), *([None] * 12)) == api.FLASHRNN_ERR_NULL
    assert api.lib().flashrnn_fwd(None, *([None] * 8)) == api.FLASHRNN_ERR_NULL
    assert api.lib().flashrnn_check(ctypes.byref(d), None, None) == api.FLASHRNN_OK


def test_sizes_and_plans_of_the_benchmark_configurations():
    from paper_2412_07752_amd import synth
    for w in synth.CONFIGS:
        d = api.make_desc(w.cell, w.T, w.B, w.NH, w.D, api.FLASHRNN_BF16 if w.dtype == "bf16" else api.FLASHRNN_F32)
        slots = {0: 4, 1: 4, 2: 8, 3: 1, 4: 4}[w.cell]   # values saved per (t, row, unit): four, the sLSTM's five padded to eight, Elman one
        assert api.flashrnn_gate_cache_bytes(d) == w.T * w.B * w.NH * w.D * slots * (2 if w.dtype == "bf16" else 4)
        assert api.flashrnn_workspace_bytes(d) > 0
        for bwd in (False, True):
            wgs, per_head, waves = api.flashrnn_plan(d, bwd)
            assert 1 <= wgs <= 256 and waves * 64 <= 1024 and per_head >= 1
    # a head that is too large for the compiled shapes is refused, not mis-run
    d = api.make_desc(0, 4, 2, 1, 4096, api.FLASHRNN_BF16)
    assert api.flashrnn_workspace_bytes(d) == 0
    # ... up to the largest fused head the paper reports (App. H.1) every multiple of 16 has a plan: beyond 1024 units
    # one workgroup per block of 16 units, spread over the whole chip
    for D in (1040, 1536, 2048, 2688):
        d = api.make_desc(0, 4, 16, 1, D, api.FLASHRNN_BF16)
        assert api.flashrnn_workspace_bytes(d) > 0
        for bwd in (False, True):
            assert api.flashrnn_plan(d, bwd)[0] % (D // 16) == 0 and api.flashrnn_plan_kernel(d, bwd)[2] == D // 16
    assert api.flashrnn_workspace_bytes(api.make_desc(0, 4, 2, 1, 2704, api.FLASHRNN_BF16)) == 0
