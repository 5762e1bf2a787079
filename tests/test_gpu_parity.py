"""GPU parity tests: the HIP path through the C ABI against the fp64 oracle, element by element,
on the same seeded inputs.  Tolerances (per output tensor, max-norm relative): 1e-5 for f32 I/O,
2e-2 for bf16 I/O plus max-abs 5e-2 on h."""
import os

import numpy as np
import pytest
import torch

import parity_util as pu
from paper_2412_07752_amd import api, synth
from paper_2412_07752_amd.synth import CELL_ELMAN, CELL_GRU, CELL_GRU4, CELL_LSTM, CELL_SLSTM, Workload

pytestmark = pytest.mark.gpu
CELLS = [CELL_LSTM, CELL_GRU, CELL_SLSTM, CELL_ELMAN, CELL_GRU4]
PLAN_ENV = ("FLASHRNN_MULTI", "FLASHRNN_BT", "FLASHRNN_NWU", "FLASHRNN_KS", "FLASHRNN_GPAR", "FLASHRNN_SPIN_LIMIT", "FLASHRNN_EBK", "FLASHRNN_DEEP_FETCH",
            "FLASHRNN_KIND", "FLASHRNN_RECOMPUTE_STEPS")


@pytest.fixture(autouse=True)
def clean_env():
    for k in PLAN_ENV:
        os.environ.pop(k, None)
    os.environ["FLASHRNN_SPIN_LIMIT"] = "400000"
    yield
    for k in PLAN_ENV:
        os.environ.pop(k, None)


def _dlast(w, seed=99):
    rng = np.random.default_rng(seed)
    return rng.standard_normal((w.S, w.B, w.NH, w.D)).astype(np.float32)


def _check(w, env=None, with_dlast=False, clip=None, elementwise=True):
    os.environ.update(env or {})
    print(f"case {w.name} env={env}", flush=True)
    inp = synth.make_inputs(w)
    dl = _dlast(w) if (with_dlast and w.backward) else None
    ref = pu.run_oracle(w, inp, dl, clip=clip)
    gpu = pu.run_gpu(w, inp, dl, clip=clip)
    res = pu.compare(w, gpu, ref)
    pu.assert_close(w, res)
    if elementwise:
        pu.assert_states_elementwise(w, gpu, ref)
    return gpu


@pytest.mark.parametrize("cell", CELLS)
@pytest.mark.parametrize("dtype,D", [("bf16", 16), ("bf16", 32), ("bf16", 48), ("bf16", 64), ("bf16", 96), ("bf16", 128),
                                     ("bf16", 160), ("bf16", 192), ("f32", 16), ("f32", 48), ("f32", 64), ("f32", 96),
                                     ("f32", 128)])
def test_one_workgroup_per_group(cell, dtype, D):
    """Ragged batch (13 rows), several heads, non-zero initial states and final-state gradients."""
    w = Workload(f"single_{cell}_{dtype}_D{D}", cell, 9, 13, 2, D, dtype, True, bias="uniform0.1", init="uniform0.1", seed=D)
    _check(w, with_dlast=True)


@pytest.mark.parametrize("cell", CELLS)
@pytest.mark.parametrize("bt", [16, 8, 4])
def test_batch_tiles(cell, bt):
    """Batch tiles of 16, 8 and 4 rows (idle MFMA lanes take over point-wise work); 21 rows = ragged last tile."""
    w = Workload(f"bt{bt}_{cell}", cell, 11, 21, 3, 64, "bf16", True, bias="forget3" if cell in (CELL_LSTM, CELL_SLSTM) else "uniform0.1",
                 init="uniform0.1", seed=bt)
    _check(w, {"FLASHRNN_BT": str(bt)}, with_dlast=True)


@pytest.mark.parametrize("cell", CELLS)
@pytest.mark.parametrize("dtype,D,env", [
    ("bf16", 64, {"FLASHRNN_NWU": "1"}), ("bf16", 64, {"FLASHRNN_NWU": "2"}), ("bf16", 128, {"FLASHRNN_NWU": "2"}),
    ("bf16", 192, {"FLASHRNN_NWU": "4"}), ("bf16", 128, {"FLASHRNN_KS": "4"}), ("bf16", 256, {}), ("bf16", 384, {}),
    ("f32", 64, {"FLASHRNN_NWU": "1"}), ("f32", 128, {"FLASHRNN_KS": "4"}), ("f32", 192, {}), ("f32", 256, {}),
])
def test_groups_split_over_workgroups(cell, dtype, D, env):
    """A head served by several workgroups that exchange h (forward) / dg (backward) every step (full 16-row tiles)."""
    e = {"FLASHRNN_MULTI": "1", "FLASHRNN_BT": "16"}
    e.update(env)
    w = Workload(f"multi_{cell}_{dtype}_D{D}", cell, 10, 19, 2, D, dtype, True, bias="uniform0.1", init="uniform0.1", seed=D + 1)
    _check(w, e, with_dlast=True)


@pytest.mark.parametrize("cell", CELLS)
@pytest.mark.parametrize("D,ebk", [(64, 1), (64, 2), (128, 1), (128, 2), (128, 4), (192, 1), (192, 3)])
def test_backward_contraction_split_over_waves(cell, D, ebk):
    """Backward tile kernel with the gate-gradient contraction in one piece per wave or split over 2, 3, 4 waves."""
    w = Workload(f"ebk{ebk}_{cell}_D{D}", cell, 8, 10, 2, D, "bf16", True, bias="uniform0.1", init="uniform0.1", seed=D + ebk)
    _check(w, {"FLASHRNN_EBK": str(ebk)}, with_dlast=True)

@pytest.mark.parametrize("cell", CELLS)
@pytest.mark.parametrize("bt", [16, 8, 4])
@pytest.mark.parametrize("D", [48, 112])
def test_batch_tiles_with_f32_io(cell, bt, D):
    """f32 I/O (f32 MFMA, rel 1e-5): the same three tile heights; 21 rows = ragged last tile, head sizes that pad the contraction axis."""
    w = Workload(f"f32_bt{bt}_{cell}_D{D}", cell, 10, 21, 2, D, "f32", True, bias="forget3" if cell in (CELL_LSTM, CELL_SLSTM) else "uniform0.1",
                 init="uniform0.1", seed=bt + D)
    _check(w, {"FLASHRNN_BT": str(bt)}, with_dlast=True)


@pytest.mark.parametrize("cell", CELLS)
@pytest.mark.parametrize("D,bt", [(32, 4), (32, 8), (64, 4), (64, 8), (16, 4), (48, 8), (48, 4)])
@pytest.mark.parametrize("T", [1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 13])
def test_backward_kernels_that_fetch_deep(cell, D, bt, T):
    """The backward kernels for inputs that come from HBM (taken by themselves only for sequences beyond the last-level cache):
    forced here on short sequences, every length around the depth of their pipeline."""
    w = Workload(f"deep_{cell}_D{D}_bt{bt}_T{T}", cell, T, 11, 2, D, "bf16", True, bias="uniform0.1", init="uniform0.1", seed=T + D + bt)
    _check(w, {"FLASHRNN_DEEP_FETCH": "1", "FLASHRNN_BT": str(bt)}, with_dlast=True)
    assert api.flashrnn_plan_kernel(api.make_desc(cell, T, 11, 2, D, api.FLASHRNN_BF16), True)[0] == 2   # (that variant ran)


@pytest.mark.parametrize("cell", CELLS)
@pytest.mark.parametrize("bt", [8, 4])
def test_generic_kernels_on_small_batch_tiles(cell, bt):
    """The generic persistent kernels (lane-wise global accesses) on the shapes the staged tile kernels normally take."""
    w = Workload(f"generic_bt{bt}_{cell}", cell, 7, 11, 2, 96, "bf16", True, bias="uniform0.1", init="uniform0.1", seed=bt + 40)
    _check(w, {"FLASHRNN_KIND": "0", "FLASHRNN_BT": str(bt)}, with_dlast=True)


@pytest.mark.parametrize("cell", CELLS)
def test_forward_only_small_batch_tile(cell):
    """No gate cache: the staged forward kernel moves states only."""
    w = Workload(f"fwdonly_{cell}", cell, 6, 7, 2, 128, "bf16", False, bias="uniform0.1", init="uniform0.1", seed=77)
    _check(w)


@pytest.mark.parametrize("cell", [CELL_LSTM, CELL_GRU, CELL_SLSTM])
def test_forward_calls_with_and_without_saved_values_plan_apart(cell):
    """More groups than CUs (12 x 64 with 256 rows): the forward call that saves its values takes 4-row tiles, the one that
    saves nothing 8-row tiles (the sLSTM 4 rows either way); both against the oracle."""
    d = api.make_desc(cell, 3, 256, 12, 64, api.FLASHRNN_BF16)
    assert api.flashrnn_plan_kernel(d, 0)[:2] == (1, 4) and api.flashrnn_plan_kernel(d, 2)[:2] == (1, 4 if cell == CELL_SLSTM else 8)
    with pytest.raises(api.FlashRNNError):
        api.flashrnn_plan_kernel(d, 3)
    for backward in (False, True):
        _check(Workload(f"twoplans_{cell}_{int(backward)}", cell, 3, 256, 12, 64, "bf16", backward, bias="uniform0.1", init="uniform0.1", seed=91))


@pytest.mark.parametrize("cell", CELLS)
@pytest.mark.parametrize("clip", [0.0, 0.02, 1e6])
@pytest.mark.parametrize("dtype,D,env", [("bf16", 64, {}), ("bf16", 192, {}), ("bf16", 96, {"FLASHRNN_KIND": "0"}), ("f32", 32, {}),
                                         ("bf16", 128, {"FLASHRNN_MULTI": "1", "FLASHRNN_KS": "4"})])
def test_recurrent_gradient_clip(cell, clip, dtype, D, env):
    """Sec. 4.1: the R^T dg_t term clipped value by value after every step (0 cuts it; a huge bound changes nothing),
    in the tile, generic, f32 and split-group kernels.  (The recurrent term has values of a few tenths here: 0.02 bites.)"""
    w = Workload(f"clip{clip}_{cell}_{dtype}_D{D}", cell, 7, 6, 2, D, dtype, True, bias="uniform0.1", init="uniform0.1", seed=D + 3)
    os.environ.update(env)
    print(f"case {w.name} env={env}", flush=True)
    inp, dl = synth.make_inputs(w), _dlast(w)
    ref, ref_free = pu.run_oracle(w, inp, dl, clip=clip), pu.run_oracle(w, inp, dl)
    gpu = pu.run_gpu(w, inp, dl, clip=clip)
    # errors relative to the scale of the unclipped gradients (the clip shrinks values, not rounding errors) ...
    res = pu.compare(w, gpu, ref, scale_ref=ref_free)
    pu.assert_close(w, res)
    # ... and with an absolute bound: the unclipped run meets the tolerance as it is defined (relative to its own
    # reference), and clipping must not make any tensor's absolute error larger than twice that run's (or than the
    # plain tolerance on the clipped reference, whichever is larger)
    gpu_free = pu.run_gpu(w, inp, dl)
    res_free = pu.compare(w, gpu_free, ref_free)
    pu.assert_close(w, res_free)
    plain = pu.compare(w, gpu, ref)
    tol = pu.TOL_BF16_REL if dtype == "bf16" else pu.TOL_F32_REL
    for k, (r, a) in plain.items():
        assert r <= tol or a <= 2.0 * res_free[k][1] + 1e-30, f"{w.name} {k}: abs {a:.3e} vs unclipped run's {res_free[k][1]:.3e}"
    if clip == 0.02:   # the bound did change the result
        assert np.abs(ref_free["dWx"] - gpu["dWx"]).max() > 1e-3


@pytest.mark.parametrize("cell", [CELL_LSTM, CELL_GRU, CELL_SLSTM])
@pytest.mark.parametrize("dtype,D", [("bf16", 208), ("bf16", 320), ("bf16", 640), ("f32", 144), ("f32", 208)])
def test_split_groups_with_padded_contraction(cell, dtype, D):
    """Head sizes between the instantiated contraction lengths: the exchanged rows and the packed R are zero beyond D."""
    w = Workload(f"pad_{cell}_{dtype}_D{D}", cell, 5, 5, 1 if D > 400 else 2, D, dtype, True, bias="uniform0.1", init="uniform0.1", seed=D)
    _check(w, with_dlast=True)


def test_largest_head_takes_a_whole_xcd():
    """D = 1024 in one head: a group is 32 workgroups (every CU of one XCD) x 2 unit waves x 4 contraction slices; the five
    batch rows make two groups of batch tile 4, on two XCDs."""
    w = Workload("lstm_D1024", CELL_LSTM, 4, 5, 1, 1024, "bf16", True, seed=9)
    _check(w)
    d = api.make_desc(CELL_LSTM, 4, 5, 1, 1024, api.FLASHRNN_BF16)
    assert api.flashrnn_plan(d)[0] == 64 and api.flashrnn_plan_kernel(d)[2] == 32


def test_backward_groups_take_whole_xcds_and_the_whole_chip_where_they_need_them():
    """A head of 1024 units needs every CU of an XCD per group in both directions (four 4-row groups of a 16-row batch side by
    side, not one 16-row group); two 8-row groups of a 2048-unit head need all 256 CUs."""
    d = api.make_desc(CELL_LSTM, 8, 16, 1, 1024, api.FLASHRNN_BF16)
    for bwd in (False, True):
        staged, bt, split = api.flashrnn_plan_kernel(d, bwd)
        assert (staged, bt, split) == (0, 4, 32) and api.flashrnn_plan(d, bwd)[0] == 128
    d = api.make_desc(CELL_LSTM, 8, 16, 1, 2048, api.FLASHRNN_BF16)
    assert api.flashrnn_plan_kernel(d, True)[1:] == (8, 128) and api.flashrnn_plan(d, True)[0] == 256
    w = Workload("lstm_D1024_B16", CELL_LSTM, 5, 16, 1, 1024, "bf16", True, bias="uniform0.1", init="uniform0.1", seed=10)
    _check(w, with_dlast=True)


@pytest.mark.parametrize("cell,D,B,NH", [(CELL_LSTM, 1040, 5, 1), (CELL_LSTM, 1280, 19, 1), (CELL_LSTM, 1536, 6, 2), (CELL_LSTM, 2048, 9, 1),
                                         (CELL_LSTM, 2688, 5, 1), (CELL_SLSTM, 1536, 7, 1), (CELL_SLSTM, 2048, 16, 1), (CELL_GRU, 1280, 12, 1),
                                         (CELL_GRU, 2688, 3, 1), (CELL_ELMAN, 2048, 4, 1), (CELL_GRU4, 1536, 4, 1)])
def test_heads_beyond_one_xcd_are_spread_over_the_chip(cell, D, B, NH):
    """Heads of more than 1024 units (App. H.1 quotes 2688 as the largest fused head on the paper's GPU): R does not fit the
    registers of one XCD's CUs, so a group's workgroups sit on all eight XCDs and exchange h / dg through memory."""
    w = Workload(f"spread_{cell}_D{D}", cell, 5, B, NH, D, "bf16", True, bias="uniform0.1", init="uniform0.1", seed=D + B)
    _check(w, with_dlast=True)
    d = api.make_desc(cell, 5, B, NH, D, api.FLASHRNN_BF16)
    for bwd in (False, True):
        assert api.flashrnn_plan_kernel(d, bwd)[2] == D // 16


@pytest.mark.parametrize("cell", CELLS)
def test_spread_groups_loop_when_they_do_not_fit(cell):
    """The spread placement forced onto a small head, two groups in flight out of nine: workgroups loop over groups."""
    w = Workload(f"spreadloop_{cell}", cell, 6, 33, 1, 64, "bf16", True, bias="uniform0.1", init="uniform0.1", seed=6)
    _check(w, {"FLASHRNN_MULTI": "2", "FLASHRNN_GPAR": "2"}, with_dlast=True)


@pytest.mark.parametrize("cell,NH,D", [(CELL_LSTM, 32, 128), (CELL_GRU, 24, 144), (CELL_SLSTM, 12, 144)])
def test_weight_gradient_gemm_with_large_tiles(cell, NH, D):
    """Many heads: the dR GEMM takes its 128 x 256 tile (ragged in both directions at D = 144; GRU: the candidate column of B comes
    from the recurrent-side gradient buffer), and the contraction over (t, b) has a ragged last round."""
    w = Workload(f"widegemm_{cell}_NH{NH}_D{D}", cell, 7, 5, NH, D, "bf16", True, bias="uniform0.1", init="uniform0.1", seed=NH + D)
    _check(w, with_dlast=True)


@pytest.mark.parametrize("cell", CELLS)
def test_group_loop_when_groups_do_not_fit(cell):
    """More groups than run at once: workgroups loop over groups and reload R per head."""
    w = Workload(f"loop_{cell}", cell, 7, 40, 3, 64, "bf16", True, bias="uniform0.1", init="uniform0.1", seed=5)
    _check(w, {"FLASHRNN_MULTI": "1", "FLASHRNN_NWU": "2", "FLASHRNN_GPAR": "4"}, with_dlast=True)


@pytest.mark.parametrize("cell", CELLS)
@pytest.mark.parametrize("T", [0, 1, 2, 3])
def test_degenerate_lengths(cell, T):
    """The staged kernels look two steps ahead: the shortest sequences take every clamped branch of that."""
    w = Workload(f"T{T}_{cell}", cell, T, 5, 2, 32, "bf16", True, bias="uniform0.1", init="uniform0.1")
    gpu = _check(w, with_dlast=True)
    if T == 0:
        assert np.all(gpu["dR"] == 0) and np.all(gpu["db"] == 0)


def test_large_single_head_split_with_contraction_slices():
    """D = 768 in one head (R is 4.7 MB): 24 workgroups x 2 unit waves x 4 contraction slices per group; with batch tiles
    of 4 rows the 16 rows make 4 groups, one per XCD."""
    w = Workload("lstm_D768", CELL_LSTM, 12, 16, 1, 768, "bf16", True, seed=3)
    _check(w)
    d = api.make_desc(CELL_LSTM, 12, 16, 1, 768, api.FLASHRNN_BF16)
    wg, per_head, waves = api.flashrnn_plan(d)
    staged, bt, split = api.flashrnn_plan_kernel(d)
    assert (wg, per_head, waves) == (96, 96, 8) and (staged, bt, split) == (False, 4, 24)
    _check(w, {"FLASHRNN_BT": "16"})
    assert api.flashrnn_plan(d) == (24, 24, 8)


@pytest.mark.parametrize("cell", CELLS)
@pytest.mark.parametrize("bt", [8, 4])
@pytest.mark.parametrize("dtype,D,env", [("bf16", 256, {}), ("bf16", 128, {"FLASHRNN_KS": "4"}), ("bf16", 64, {"FLASHRNN_NWU": "1"})])
def test_split_groups_on_small_batch_tiles(cell, bt, dtype, D, env):
    """A head split over workgroups with batch tiles of 8 and 4 rows: fewer rows to exchange per group, lanes collect the four
    units of an exchange word from their neighbours before publishing."""
    e = {"FLASHRNN_MULTI": "1", "FLASHRNN_BT": str(bt)}
    e.update(env)
    w = Workload(f"multibt{bt}_{cell}_D{D}", cell, 9, 13, 2, D, dtype, True, bias="uniform0.1", init="uniform0.1", seed=D + bt)
    _check(w, e, with_dlast=True)


LARGE_CASES = [
    # (dtype, D, environment, batch): staged tile kernels, generic kernels, a head split over workgroups (with and
    # without contraction slices), f32 single and split
    ("bf16", 64, {}, 13), ("bf16", 192, {}, 6), ("bf16", 96, {"FLASHRNN_KIND": "0", "FLASHRNN_BT": "4"}, 9),
    ("bf16", 64, {"FLASHRNN_BT": "16"}, 19), ("bf16", 256, {}, 7), ("bf16", 128, {"FLASHRNN_MULTI": "1", "FLASHRNN_KS": "4"}, 18),
    ("f32", 64, {}, 5), ("f32", 192, {}, 6),
]


@pytest.mark.parametrize("cell", CELLS)
@pytest.mark.parametrize("init", ["uniform0.1_bounded", "zero"])
@pytest.mark.parametrize("dtype,D,env,B", LARGE_CASES)
def test_saturated_gates(cell, init, dtype, D, env, B):
    """Finite pre-activations far out in both tails (a third of all Wx entries shifted by +-50, +-100, +-200, on every
    gate), non-zero R, 12 steps so that the sLSTM stabilizer is carried through jumps in both directions: the regime m
    exists for (App. A).  Nothing may overflow, underflow into a wrong branch or turn into NaN, forward or backward.
    Non-zero initial states respect the cell's invariant |c| <= n (|h| <= 1): bf16 rounding of an h of 100 and more would
    move pre-activations by tenths.  With f32 I/O the element-wise check of the sLSTM states is left to the max-norm one:
    the stabilizer reaches 230 here, where one float32 ulp is 1.5e-5, and every weight exp(. - m) carries that as a
    relative error, so single elements sit at 1e-5 to 2e-5."""
    w = Workload(f"sat_{cell}_{dtype}_D{D}_{init}", cell, 12, B, 2, D, dtype, True, bias="forget3" if cell in (CELL_LSTM, CELL_SLSTM) else "uniform0.1",
                 init=init, seed=D + B, wx="large_mix")
    gpu = _check(w, env, with_dlast=True, elementwise=not (cell == CELL_SLSTM and dtype == "f32"))
    for k, v in gpu.items():
        assert np.all(np.isfinite(v)), k


def test_forward_timeout_survives_the_backward_call():
    """A split plan whose forward waits gave up: the backward call that follows runs with a normal limit, and one check
    after it still reports the forward timeout (the two passes keep separate error words; only a forward call clears both)."""
    w = Workload("sticky", CELL_LSTM, 6, 16, 1, 64, "bf16", True)
    inp = synth.make_inputs(w)
    os.environ.update({"FLASHRNN_MULTI": "1", "FLASHRNN_NWU": "1", "FLASHRNN_SPIN_LIMIT": "-1"})
    Wx, R, b, dH = (pu.to_device(inp[k], "bf16") for k in ("Wx", "R", "b", "dH"))
    desc = api.make_desc(w.cell, w.T, w.B, w.NH, w.D, api.FLASHRNN_BF16)
    states, cache, ws = api.flashrnn_fwd(w.cell, Wx, R, b)
    os.environ["FLASHRNN_SPIN_LIMIT"] = "400000"
    api.flashrnn_bwd(w.cell, R, b, states, cache, dH, workspace=ws)
    with pytest.raises(api.FlashRNNError) as ei:
        api.flashrnn_check(desc, ws)
    assert ei.value.status == api.FLASHRNN_ERR_TIMEOUT
    # the next forward / backward pair on the same workspace is clean and correct again
    ref = pu.run_oracle(w, inp)
    states, cache, ws = api.flashrnn_fwd(w.cell, Wx, R, b, workspace=ws)
    dWx, dR, db, ds0 = api.flashrnn_bwd(w.cell, R, b, states, cache, dH, workspace=ws)
    api.flashrnn_check(desc, ws)
    gpu = {"states": pu.to_host64(states), "dWx": pu.to_host64(dWx), "dR": pu.to_host64(dR), "db": pu.to_host64(db), "dstates0": pu.to_host64(ds0)}
    pu.assert_close(w, pu.compare(w, gpu, ref))


def test_seeded_random_shapes():
    """A seeded sweep over (cell, dtype, T, B, NH, D, forward-only / backward, clip, initial states, final-state gradients)
    with whatever plan the library picks for each shape; stops at the first mismatch and names the case."""
    import random
    rng = random.Random(20241207)
    for it in range(48):
        cell = rng.choice(CELLS)
        dtype = rng.choice(["bf16", "bf16", "bf16", "f32"])
        D = 16 * rng.choice([1, 2, 3, 4, 5, 6, 8, 9, 10, 12, 16, 20, 24] if dtype == "bf16" else [1, 2, 3, 4, 6, 8, 12, 16])
        NH = rng.choice([1, 2, 3, 5, 8, 20])
        B = rng.choice([1, 2, 3, 4, 5, 7, 8, 9, 16, 17, 33, 64])
        T = rng.choice([1, 2, 3, 4, 5, 8, 13])
        while NH * B * D * T > 400000 and B > 1:
            B = max(1, B // 2)
        bw = rng.random() < 0.8
        clip = rng.choice([None, None, 0.05, 0.0]) if bw else None
        w = Workload(f"rand{it}", cell, T, B, NH, D, dtype, bw, bias="uniform0.1", init=rng.choice(["zero", "uniform0.1"]), seed=it + 1000)
        print(f"case {it}: cell {cell} {dtype} T {T} B {B} NH {NH} D {D} bwd {bw} clip {clip}", flush=True)
        inp = synth.make_inputs(w)
        dl = _dlast(w, seed=it) if (bw and rng.random() < 0.5) else None
        ref = pu.run_oracle(w, inp, dl, clip=clip)
        free = pu.run_oracle(w, inp, dl) if clip is not None else None
        gpu = pu.run_gpu(w, inp, dl, clip=clip)
        pu.assert_close(w, pu.compare(w, gpu, ref, scale_ref=free))
        pu.assert_states_elementwise(w, gpu, ref)


RECOMPUTE_CASES = [
    # (dtype, D, B, T, environment): staged tile kernels, generic kernels, a head split over workgroups, f32; windows of 4 steps
    # (T = 11: a ragged first window), of one step, and the whole sequence in one window
    ("bf16", 64, 13, 11, {"FLASHRNN_RECOMPUTE_STEPS": "4"}), ("bf16", 192, 6, 9, {"FLASHRNN_RECOMPUTE_STEPS": "1"}),
    ("bf16", 96, 19, 11, {"FLASHRNN_RECOMPUTE_STEPS": "4", "FLASHRNN_KIND": "0", "FLASHRNN_BT": "16"}), ("bf16", 256, 7, 11, {"FLASHRNN_RECOMPUTE_STEPS": "3"}),
    ("bf16", 80, 5, 7, {}), ("f32", 48, 9, 10, {"FLASHRNN_RECOMPUTE_STEPS": "4"}), ("f32", 192, 5, 6, {"FLASHRNN_RECOMPUTE_STEPS": "2"}),
    # ... and the backward kernels that fetch deep, in windows of 5 steps (a ragged first window of 3)
    ("bf16", 64, 13, 13, {"FLASHRNN_RECOMPUTE_STEPS": "5", "FLASHRNN_DEEP_FETCH": "1"}),
]


@pytest.mark.parametrize("cell", CELLS)
@pytest.mark.parametrize("dtype,D,B,T,env", RECOMPUTE_CASES)
def test_backward_with_recomputed_values(cell, dtype, D, B, T, env):
    """flashrnn_bwd_recompute: forward without a gate cache, backward from Wx and the states alone, window by window
    (carried state gradients, db sums and the GRU's recurrent-side gradients cross the window boundaries)."""
    os.environ.update(env)
    w = Workload(f"recompute_{cell}_{dtype}_D{D}", cell, T, B, 2, D, dtype, True, bias="uniform0.1", init="uniform0.1", seed=D + T)
    print(f"case {w.name} env={env}", flush=True)
    inp, dl = synth.make_inputs(w), _dlast(w)
    ref = pu.run_oracle(w, inp, dl)
    Wx, R, b, dH = (pu.to_device(inp[k], dtype) for k in ("Wx", "R", "b", "dH"))
    s0, dlast = pu.to_device(inp["states0"], "f32"), pu.to_device(dl, "f32")
    states, cache, ws = api.flashrnn_fwd(cell, Wx, R, b, s0, save_for_backward=False)
    assert cache is None
    dWx, dR, db, ds0, ws2 = api.flashrnn_bwd_recompute(cell, Wx, R, b, states, dH, dlast)
    desc = api.make_desc(cell, T, B, 2, D, api.FLASHRNN_BF16 if dtype == "bf16" else api.FLASHRNN_F32)
    api.flashrnn_check(desc, ws2)
    gpu = {"states": pu.to_host64(states), "dWx": pu.to_host64(dWx), "dR": pu.to_host64(dR), "db": pu.to_host64(db), "dstates0": pu.to_host64(ds0)}
    pu.assert_close(w, pu.compare(w, gpu, ref))


def test_backward_with_recomputed_values_empty_sequence():
    w = Workload("recompute_T0", CELL_SLSTM, 0, 5, 2, 32, "bf16", True, bias="uniform0.1", init="uniform0.1")
    inp, dl = synth.make_inputs(w), _dlast(w)
    ref = pu.run_oracle(w, inp, dl)
    Wx, R, b, dH = (pu.to_device(inp[k], "bf16") for k in ("Wx", "R", "b", "dH"))
    states, _, _ = api.flashrnn_fwd(w.cell, Wx, R, b, pu.to_device(inp["states0"], "f32"), save_for_backward=False)
    dWx, dR, db, ds0, _ = api.flashrnn_bwd_recompute(w.cell, Wx, R, b, states, dH, pu.to_device(dl, "f32"))
    gpu = {"states": pu.to_host64(states), "dWx": pu.to_host64(dWx), "dR": pu.to_host64(dR), "db": pu.to_host64(db), "dstates0": pu.to_host64(ds0)}
    pu.assert_close(w, pu.compare(w, gpu, ref))


def test_runs_are_bitwise_reproducible():
    """No float atomics anywhere: two runs give identical bits (single and split groups)."""
    for env in ({}, {"FLASHRNN_MULTI": "1", "FLASHRNN_NWU": "1"}):
        os.environ.update(env)
        w = Workload("repro", CELL_SLSTM, 16, 16, 2, 64, "bf16", True, bias="forget3", init="uniform0.1")
        inp = synth.make_inputs(w)
        a = pu.run_gpu(w, inp)
        b = pu.run_gpu(w, inp)
        for k in a:
            assert np.array_equal(a[k], b[k]), k


def test_chunked_sequence_equals_one_call():
    """states0 in / last states out: T1 steps then T2 steps from the saved states == T1 + T2 steps (f32 path, exact)."""
    w = Workload("chunk", CELL_SLSTM, 12, 8, 2, 32, "f32", False, bias="forget3", init="uniform0.1")
    inp = synth.make_inputs(w)
    Wx, R, b = (pu.to_device(inp[k], "f32") for k in ("Wx", "R", "b"))
    s0 = pu.to_device(inp["states0"], "f32")
    full, _, _ = api.flashrnn_fwd(w.cell, Wx, R, b, s0, save_for_backward=False)
    a, _, _ = api.flashrnn_fwd(w.cell, Wx[:7].contiguous(), R, b, s0, save_for_backward=False)
    c, _, _ = api.flashrnn_fwd(w.cell, Wx[7:].contiguous(), R, b, a[7].contiguous(), save_for_backward=False)
    torch.cuda.synchronize()
    assert torch.equal(torch.cat([a, c[1:]]), full)


def test_exchange_timeout_is_reported_not_hung():
    """Negative spin limit: every cross-CU wait gives up at once, every kernel still runs to its end,
    flashrnn_check reports the timeout, and the next call with a normal limit is correct again."""
    w = Workload("timeout", CELL_LSTM, 6, 16, 1, 64, "bf16", False)
    inp = synth.make_inputs(w)
    os.environ.update({"FLASHRNN_MULTI": "1", "FLASHRNN_NWU": "1", "FLASHRNN_SPIN_LIMIT": "-1"})
    with pytest.raises(api.FlashRNNError) as ei:
        pu.run_gpu(w, inp)
    assert ei.value.status == api.FLASHRNN_ERR_TIMEOUT
    os.environ["FLASHRNN_SPIN_LIMIT"] = "400000"
    ref = pu.run_oracle(w, inp)
    pu.assert_close(w, pu.compare(w, pu.run_gpu(w, inp), ref))


def test_binding_rejects_wrong_shapes_and_dtypes():
    dev = "cuda"
    Wx = torch.zeros((4, 2, 4, 1, 32), dtype=torch.bfloat16, device=dev)
    R = torch.zeros((1, 32, 4, 32), dtype=torch.bfloat16, device=dev)
    b = torch.zeros((1, 4, 32), dtype=torch.bfloat16, device=dev)
    with pytest.raises(ValueError):
        api.flashrnn_fwd(CELL_LSTM, Wx, R[:, :16].contiguous(), b)
    with pytest.raises(ValueError):
        api.flashrnn_fwd(CELL_LSTM, Wx, R.float(), b)
    with pytest.raises(ValueError):
        api.flashrnn_fwd(CELL_GRU, Wx, R, b)
    with pytest.raises(TypeError):
        api.flashrnn_fwd(CELL_LSTM, Wx.half(), R.half(), b.half())
    ws = torch.empty(1 << 20, dtype=torch.uint8, device=dev)
    d = api.make_desc(CELL_LSTM, 4, 2, 1, 32, api.FLASHRNN_BF16)
    import ctypes
    st = torch.empty((5, 2, 2, 1, 32), dtype=torch.float32, device=dev)
    rc = api.lib().flashrnn_fwd(ctypes.byref(d), Wx.data_ptr(), R.data_ptr(), b.data_ptr(), None, st.data_ptr(), None,
                                ws.data_ptr() + 8, None)
    assert rc == api.FLASHRNN_ERR_WORKSPACE


@pytest.mark.parametrize("D", [64, 256])
def test_forward_backward_replay_from_a_hip_graph(D):
    """The two entry points allocate nothing and record only kernels, so a caller may capture them.  The graph is replayed
    several times, with eager work and synchronizations in between, on changing inputs; every replay must reproduce the eager
    result bit for bit (one workgroup per group, and a head split over workgroups with its exchange buffers)."""
    w = Workload(f"graph_D{D}", CELL_SLSTM, 12, 8, 2, D, "bf16", True, bias="forget3", init="uniform0.1", seed=D)
    inp = synth.make_inputs(w)
    Wx, R, b = (pu.to_device(inp[k], "bf16") for k in ("Wx", "R", "b"))
    s0, dH = pu.to_device(inp["states0"], "f32"), pu.to_device(inp["dH"], "bf16")
    desc = api.make_desc(w.cell, w.T, w.B, w.NH, w.D, api.FLASHRNN_BF16)
    ws = api.alloc_workspace(desc, "cuda")
    states = torch.empty((w.T + 1, w.S, w.B, w.NH, w.D), dtype=torch.float32, device="cuda")
    cache = torch.empty(api.flashrnn_gate_cache_bytes(desc), dtype=torch.uint8, device="cuda")
    out = (torch.empty((w.T, w.B, w.G, w.NH, w.D), dtype=torch.bfloat16, device="cuda"), torch.empty((w.NH, w.D, w.G, w.D), device="cuda"),
           torch.empty((w.NH, w.G, w.D), device="cuda"), torch.empty((w.S, w.B, w.NH, w.D), device="cuda"))

    def step():
        api.flashrnn_fwd(w.cell, Wx, R, b, s0, workspace=ws, states=states, gate_cache=cache)
        api.flashrnn_bwd(w.cell, R, b, states, cache, dH, None, workspace=ws, out=out)

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in (states,) + out]

    step()                       # warm-up outside the capture (kernel attributes are set on first use)
    api.flashrnn_check(desc, ws)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(3):
        Wx.copy_(torch.roll(Wx, 1, dims=0))          # new inputs, same buffers
        dH.mul_(-1.0)
        step()
        eager = snapshot()
        for t in (states,) + out:
            t.fill_(float("nan"))
        graph.replay()
        replayed = snapshot()
        api.flashrnn_check(desc, ws)
        for a, r in zip(eager, replayed):
            assert torch.equal(a, r), f"replay {rep} differs from the eager result"
