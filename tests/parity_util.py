"""Helpers of the GPU parity tests: run one workload through the oracle (fp64, CPU) and through the
C-ABI library (GPU) on the same seeded inputs, and measure the differences.

Error measure per output tensor: max|gpu - ref| / max(max|ref|, tiny)  ("rel"), and max|gpu - ref| ("abs").
The states are checked element by element as well: |gpu - ref| <= rel_tol * (|ref| + rms(ref)), so that a small
element is not hidden behind the tensor's largest value.
"""
import numpy as np
import torch

import oracle
from paper_2412_07752_amd import api, synth

# spec tolerances
TOL_F32_REL = 1e-5
TOL_BF16_REL = 2e-2
TOL_BF16_ABS_H = 5e-2


def to_device(a, dtype):
    """float32 numpy array (already representable in the I/O dtype) -> device tensor of that dtype."""
    if a is None:
        return None
    if dtype == "bf16":
        bits = synth.bf16_bits(a)
        return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def to_host64(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def err(gpu, ref):
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0, 0.0
    d = float(np.max(np.abs(gpu - ref)))
    if not np.isfinite(d):
        return float("inf"), float("inf")
    return d / max(float(np.max(np.abs(ref))), 1e-30), d


def run_oracle(w, inp, dstates_last=None, clip=None):
    f64 = lambda a: None if a is None else a.astype(np.float64)
    st = oracle.fwd(w.cell, f64(inp["Wx"]), f64(inp["R"]), f64(inp["b"]), f64(inp["states0"]))
    out = {"states": st}
    if w.backward:
        dWx, dR, db, ds0 = oracle.bwd(w.cell, f64(inp["Wx"]), f64(inp["R"]), f64(inp["b"]), st, f64(inp["dH"]), f64(dstates_last),
                                      recurrent_clip=clip)
        out.update(dWx=dWx, dR=dR, db=db, dstates0=ds0)
    return out


def run_gpu(w, inp, dstates_last=None, check=True, clip=None):
    """clip: the oracle's convention (None off, c >= 0 bound, 0 = cut); the C ABI spells it 0 / c / negative."""
    Wx, R, b = (to_device(inp[k], w.dtype) for k in ("Wx", "R", "b"))
    s0 = to_device(inp["states0"], "f32")
    states, cache, ws = api.flashrnn_fwd(w.cell, Wx, R, b, s0, save_for_backward=w.backward)
    desc = api.make_desc(w.cell, w.T, w.B, w.NH, w.D, api.FLASHRNN_BF16 if w.dtype == "bf16" else api.FLASHRNN_F32)
    if check:
        api.flashrnn_check(desc, ws)
    out = {"states": to_host64(states)}
    if w.backward:
        dH = to_device(inp["dH"], w.dtype)
        dl = to_device(dstates_last, "f32")
        gclip = 0.0 if clip is None else (-1.0 if clip == 0 else float(clip))
        dWx, dR, db, ds0 = api.flashrnn_bwd(w.cell, R, b, states, cache, dH, dl, workspace=ws, recurrent_grad_clip=gclip)
        if check:
            api.flashrnn_check(desc, ws)
        out.update(dWx=to_host64(dWx), dR=to_host64(dR), db=to_host64(db), dstates0=to_host64(ds0))
    torch.cuda.synchronize()
    return out


def compare(w, gpu, ref, scale_ref=None):
    """dict name -> (rel, abs); states are split per state so that a small state is not hidden by a large one.
    scale_ref (another reference result): the error is taken relative to the larger of the two references' maxima.
    A clipped gradient is compared that way, against the scale of the unclipped one: the clip shrinks the values,
    not the rounding error of the terms below the bound."""
    res = {}
    names = "hcnm"
    for s in range(w.S):
        res[f"states.{names[s]}"] = err(gpu["states"][:, s], ref["states"][:, s])
    for k in ("dWx", "dR", "db"):
        if k in ref:
            res[k] = err(gpu[k], ref[k])
    if "dstates0" in ref:
        for s in range(w.S):
            res[f"dstates0.{names[s]}"] = err(gpu["dstates0"][s], ref["dstates0"][s])
    if scale_ref is not None:
        for k, (r, a) in list(res.items()):
            base, idx = (k.split(".") + [None])[:2]
            pick = (lambda d: d[base]) if idx is None else (lambda d: d[base][:, names.index(idx)] if base == "states" else d[base][names.index(idx)])
            m = max(np.abs(pick(ref)).max(initial=0.0), np.abs(pick(scale_ref)).max(initial=0.0))
            res[k] = (a / m if m > 0 else r, a)
    return res


def assert_states_elementwise(w, gpu, ref):
    """Per element and state: |gpu - ref| <= rel_tol * (|ref| + rms(ref))."""
    rel = TOL_BF16_REL if w.dtype == "bf16" else TOL_F32_REL
    for s in range(w.S):
        g, r = np.asarray(gpu["states"][:, s], dtype=np.float64), np.asarray(ref["states"][:, s], dtype=np.float64)
        if r.size == 0:
            continue
        bound = rel * (np.abs(r) + np.sqrt(np.mean(r * r)))
        bad = np.abs(g - r) > bound
        assert not bad.any(), f"{w.name} states.{'hcnm'[s]}: {int(bad.sum())} of {r.size} elements off, worst " \
                              f"{float(np.max(np.abs(g - r) / np.maximum(bound, 1e-300))):.2f} x bound"


def assert_close(w, res):
    rel = TOL_BF16_REL if w.dtype == "bf16" else TOL_F32_REL
    for k, (r, a) in res.items():
        assert np.isfinite(r), f"{w.name} {k}: non-finite"
        # a reference that is identically zero (e.g. dstates0 of the stabilizer) must be matched exactly
        assert r <= rel or a == 0.0, f"{w.name} {k}: rel {r:.3e} abs {a:.3e} > {rel}"
    if w.dtype == "bf16":
        # max-abs 5e-2 on h is meant for h in its natural range |h| <= 1; initial states a caller passes in can push the
        # sLSTM's h = o c / n beyond it (|c_0| > n_0), and the bound then scales with max|h|
        r, a = res["states.h"]
        h_max = a / r if r > 0 else 0.0
        assert a <= TOL_BF16_ABS_H * max(1.0, h_max), f"{w.name} h: abs {a:.3e} (max|h| {h_max:.3g})"
