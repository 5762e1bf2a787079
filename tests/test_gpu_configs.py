"""The five benchmark configurations at full size, in the launch configuration bench.py times.

C1-C4: every output element against the oracle in one oracle call.  C5 (0.8 TFLOP in fp64, 15 GB of float64
buffers in one piece): the GPU runs the whole problem once; the oracle runs head after head (heads are
independent, so a head's slice of every output is computed exactly, including dR/db which sum over the
whole batch and all steps), all eight of them: every output element is compared."""
import numpy as np
import pytest

import parity_util as pu
from paper_2412_07752_amd import api, synth

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("idx", [0, 1, 2, 3])
def test_config_full_size(idx):
    w = synth.CONFIGS[idx]
    print(f"config {w.name}", flush=True)
    inp = synth.make_inputs(w)
    ref = pu.run_oracle(w, inp)
    gpu = pu.run_gpu(w, inp)
    res = pu.compare(w, gpu, ref)
    print({k: f"{r:.2e}/{a:.2e}" for k, (r, a) in res.items()}, flush=True)
    pu.assert_close(w, res)
    pu.assert_states_elementwise(w, gpu, ref)


def test_config5_full_size_every_head_against_oracle():
    w = synth.CONFIGS[4]
    print(f"config {w.name}: drawing inputs", flush=True)
    inp = synth.make_inputs(w)
    print("running GPU", flush=True)
    gpu = pu.run_gpu(w, inp)
    for n in range(w.NH):
        print(f"oracle on head {n}", flush=True)
        sub = synth.Workload(f"{w.name}_head{n}", w.cell, w.T, w.B, 1, w.D, w.dtype, True)
        sinp = {"Wx": np.ascontiguousarray(inp["Wx"][:, :, :, n:n + 1]), "R": inp["R"][n:n + 1], "b": inp["b"][n:n + 1],
                "states0": np.ascontiguousarray(inp["states0"][:, :, n:n + 1]), "dH": np.ascontiguousarray(inp["dH"][:, :, n:n + 1])}
        ref = pu.run_oracle(sub, sinp)
        g = {"states": gpu["states"][:, :, :, n:n + 1], "dWx": gpu["dWx"][:, :, :, n:n + 1], "dR": gpu["dR"][n:n + 1],
             "db": gpu["db"][n:n + 1], "dstates0": gpu["dstates0"][:, :, n:n + 1]}
        res = pu.compare(sub, g, ref)
        print({k: f"{r:.2e}/{a:.2e}" for k, (r, a) in res.items()}, flush=True)
        pu.assert_close(sub, res)
        pu.assert_states_elementwise(sub, g, ref)


@pytest.mark.gpu
def test_headline_workload_runs_on_the_staged_kernels():
    """The planner refuses kernels that spill registers (known only with a device).  The staged kernels of the headline
    workload sit a register or two below their budget: if a change makes one of them spill, the planner silently falls
    back to the generic kernel, which is 1.5x to 2x slower.  This test makes that loud."""
    w = synth.CONFIGS[1]
    d = api.make_desc(w.cell, w.T, w.B, w.NH, w.D, api.FLASHRNN_BF16)
    for bwd in (False, True):
        staged, bt, split = api.flashrnn_plan_kernel(d, bwd)
        assert staged and bt == 4 and split == 1, (bwd, staged, bt, split)
