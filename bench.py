"""Benchmark of the FlashRNN hot path on one MI355X.

A "step" is one pass of the whole hot path -- flashrnn_fwd followed by flashrnn_bwd (time loop in
both directions, dR GEMM, db reduction) -- over one batch of synthetic input, by default the
configuration the headline metric is quoted on (sLSTM, B=16, T=256, NH=4, D=192, bf16 I/O with f32
states).  Inputs are resident in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload IDX] [--no-cpu-baseline]
    python bench.py --copy-calibration     # a plain copy of known size, for scaling rocprofv3's HBM counters
    python bench.py --shape slstm,1024,16,4,192   # any (cell, T, B, NH, D) of the paper's sweeps; add ",fwd" for forward only
    python bench.py --sweep [--sweep-out FILE]    # the paper's runtime sweeps (Sec. 6.1, App. H.3/H.5) in one run, as a table
    python bench.py --workload 4 --recompute      # backward pass without saved values (flashrnn_bwd_recompute)
    python bench.py --workload 4 --trace-phases   # per-phase clocks of a time step (split-group kernels; needs the trace build:
                                                  # python -m paper_2412_07752_amd.build --trace), printed instead of the bench line

The `roofline` object (dominant kernel = the longer of the two persistent time-loop kernels):
  bound      the roofline that binds by arithmetic intensity: flops / algorithmic bytes against the ridge
             (2500 TFLOP/s / 8 TB/s = 312 flop/B for bf16): "hbm" for every workload here
  achieved   algorithmic bytes per launch / mean launch duration (HIP events on the dispatch), GB/s;  peak 8000 GB/s
  algorithmic bytes per (b, t) pair, H = NH*D, e = bytes of the I/O dtype:
             forward   G*H*e (Wx) + S*H*4 (states) + G*H*e (values saved for the backward pass; 0 in a forward-only call)
             backward  G*H*e (saved values) + S*H*4 (states) + H*e (dH) + G*H*e (dWx)
  traffic    HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled by a copy kernel of known
             size), read from profiles/counters_<workload>.txt -- only if that file was taken with the same launch plan as
             this run's (its plan_signature line), else null; traffic_source names the file and the commit it was taken at
  kernels    per time-loop kernel the three fractions with their denominators: recurrent-product flops against the whole
             device's MFMA peak, against the peak of the CUs the launch occupies (useful flops only: padded batch columns
             of an MFMA tile do not count), and algorithmic bytes against the HBM peak
  mfma_pipe_busy_share  share of the kernel's duration in which a SIMD's matrix pipe is busy (SQ_VALU_MFMA_BUSY_CYCLES),
             from the same counters file; it counts padded columns too and is NOT a utilisation of useful flops
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_MFMA_TFLOPS = 2500.0   # MI355X dense bf16
PEAK_F32_MFMA_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0
DEVICE_CUS = 256


def plan_call(bwd, backward):
    """Which call's plan to ask the library for: the backward call (1), the forward call of a workload with a backward pass
    (0: it saves its values) or the forward call of a forward-only workload (2: it saves nothing)."""
    return 1 if bwd else (0 if backward else 2)


def plan_signature(api, desc, backward):
    """One line that names the launch plans of a descriptor: what a counters file must match to be quoted."""
    parts = []
    for bwd in ([False, True] if backward else [False]):
        wgs, per_head, waves = api.flashrnn_plan(desc, plan_call(bwd, backward))
        staged, bt, split = api.flashrnn_plan_kernel(desc, plan_call(bwd, backward))
        parts.append(f"{'bwd' if bwd else 'fwd'}:wgs={wgs},waves={waves},staged={int(staged)},bt={bt},split={split}")
    return " ".join(parts)


def algorithmic_bytes(w, esz, backward_kernel, saves):
    """Bytes per launch of a time-loop kernel by the per-(b,t) formula in the module docstring."""
    H = w.NH * w.D
    if backward_kernel:
        per = w.G * H * esz + w.S * H * 4 + H * esz + w.G * H * esz
    else:
        per = w.G * H * esz + w.S * H * 4 + (w.G * H * esz if saves else 0)
    return per * w.B * w.T


class Runner:
    """Device buffers of one workload and the timed loop over the C-ABI calls."""

    def __init__(self, w, tensors, api, torch, recompute=False):
        self.w, self.api, self.torch = w, api, torch
        self.recompute = recompute and w.backward
        self.Wx, self.R, self.b, self.s0, self.dH = tensors
        bf16 = w.dtype == "bf16"
        self.desc = api.make_desc(w.cell, w.T, w.B, w.NH, w.D, api.FLASHRNN_BF16 if bf16 else api.FLASHRNN_F32)
        self.ws = api.alloc_workspace(self.desc, "cuda")
        if self.recompute:   # backward without saved values: the workspace also holds one window of re-formed values
            import ctypes
            self.ws = torch.zeros(api.lib().flashrnn_recompute_workspace_bytes(ctypes.byref(self.desc)), dtype=torch.uint8, device="cuda")
        T, B, NH, D, G, S = w.T, w.B, w.NH, w.D, w.G, w.S
        self.states = torch.empty((T + 1, S, B, NH, D), dtype=torch.float32, device="cuda")
        self.cache = torch.empty(max(api.flashrnn_gate_cache_bytes(self.desc), 16), dtype=torch.uint8, device="cuda") if (w.backward and not self.recompute) else None
        io_dt = torch.bfloat16 if bf16 else torch.float32
        self.out = None
        if w.backward:
            self.out = (torch.empty((T, B, G, NH, D), dtype=io_dt, device="cuda"), torch.empty((NH, D, G, D), dtype=torch.float32, device="cuda"),
                        torch.empty((NH, G, D), dtype=torch.float32, device="cuda"), torch.empty((S, B, NH, D), dtype=torch.float32, device="cuda"))

    def step(self):
        w, api = self.w, self.api
        api.flashrnn_fwd(w.cell, self.Wx, self.R, self.b, self.s0, save_for_backward=w.backward and not self.recompute, workspace=self.ws,
                         states=self.states, gate_cache=self.cache)
        if self.recompute:
            api.flashrnn_bwd_recompute(w.cell, self.Wx, self.R, self.b, self.states, self.dH, None, workspace=self.ws, out=self.out)
        elif w.backward:
            api.flashrnn_bwd(w.cell, self.R, self.b, self.states, self.cache, self.dH, None, workspace=self.ws, out=self.out)

    def run(self, steps, warmup):
        """Returns (ms per step, forward kernel ms, backward kernel ms, launches timed)."""
        api, torch = self.api, self.torch
        for _ in range(warmup):
            self.step()
        torch.cuda.synchronize()
        api.flashrnn_check(self.desc, self.ws)      # a cross-CU wait that gave up would make the numbers meaningless
        # HIP events on the persistent kernels' own dispatches, on about 25 calls spread over the timed region (a dispatch
        # that carries events starts ~5 us late: on every call that would be 1.7 % of the headline step)
        api.flashrnn_profile_enable(max(1, steps // 25))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            self.step()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        fwd_ms, nf = api.flashrnn_profile_kernel_ms(False)
        bwd_ms, nb = api.flashrnn_profile_kernel_ms(True) if self.w.backward else (0.0, 0)
        api.flashrnn_profile_enable(False)
        api.flashrnn_check(self.desc, self.ws)
        return (t1 - t0) * 1e3 / steps, fwd_ms, bwd_ms, nf


def draw_on_device(torch, synth, cell, T, B, NH, D, backward, name):
    """bf16 workload with the paper's recipe (Wx, dH ~ N(0,1), R ~ N(0,1/D), forget bias 3), drawn on the GPU."""
    w = synth.Workload(name, cell, T, B, NH, D, "bf16", backward)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(0)
    Wx = torch.randn((T, B, w.G, NH, D), device="cuda", generator=gen).bfloat16()
    R = (torch.randn((NH, D, w.G, D), device="cuda", generator=gen) / D ** 0.5).bfloat16()
    b = torch.zeros((NH, w.G, D), device="cuda")
    if cell in (synth.CELL_LSTM, synth.CELL_SLSTM):
        b[:, synth.FORGET_GATE] = 3.0
    dH = torch.randn((T, B, NH, D), device="cuda", generator=gen).bfloat16() if backward else None
    return w, (Wx, R, b.bfloat16(), None, dH)


def sweep(args, torch, api, synth):
    """The runtime sweeps of Sec. 6.1 (Figures 2-4: head size at d = 768, batch size at 12 x 64 and 1 x 768) and App. H.3 / H.5
    (sequence length; the same for the sLSTM), forward and forward + backward, plus the heads beyond one XCD (App. H.1)."""
    rows = []
    shapes = []
    for NH, D in ((48, 16), (24, 32), (12, 64), (6, 128), (4, 192), (3, 256), (2, 384), (1, 768)):
        shapes.append(("head size, d=768 B=16 T=1024", 1024, 16, NH, D))
    for NH, D in ((12, 64), (1, 768)):
        for B in (2, 4, 8, 16, 32, 64, 128, 256):
            shapes.append((f"batch size, {NH}x{D} T=1024", 1024, B, NH, D))
        for T in (256, 512, 1024, 2048):
            shapes.append((f"sequence length, {NH}x{D} B=16", T, 16, NH, D))
    for D in (1536, 2048, 2688):
        shapes.append(("one large head, B=16 T=256", 256, 16, 1, D))
    out = open(args.sweep_out, "w") if args.sweep_out else None

    def emit(line):
        print(line, flush=True)
        if out:
            out.write(line + "\n")
            out.flush()

    emit("# sweep | cell | T | B | NH | D | fwd-only ms | fwd+bwd ms | fwd kernel ms | bwd kernel ms | B*T steps/s (fwd+bwd) | plan fwd / bwd "
         "(workgroups, staged, batch tile, workgroups per group)")
    for cell in (synth.CELL_LSTM, synth.CELL_SLSTM):
        for label, T, B, NH, D in shapes:
            res = {}
            for backward in (False, True):
                w, tensors = draw_on_device(torch, synth, cell, T, B, NH, D, backward, "sweep")
                r = Runner(w, tensors, api, torch)
                steps = 3 if B * T * NH * D >= 64 * 1024 * 768 else 10
                ms, fwd_ms, bwd_ms, _ = r.run(steps, 2)
                res[backward] = (ms, fwd_ms, bwd_ms)
                if backward:
                    plans = []
                    for bwd in (False, True):
                        staged, bt, split = api.flashrnn_plan_kernel(r.desc, bwd)
                        plans.append(f"{api.flashrnn_plan(r.desc, bwd)[0]},{int(staged)},{bt},{split}")
                del r, tensors
                torch.cuda.empty_cache()
            ms_fb = res[True][0]
            emit(f"{label} | {synth.CELL_NAMES[cell]} | {T} | {B} | {NH} | {D} | {res[False][0]:.3f} | {ms_fb:.3f} | {res[True][1]:.3f} | "
                 f"{res[True][2]:.3f} | {B * T / (ms_fb * 1e-3):.3e} | {' / '.join(plans)}")
    if out:
        out.close()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=25)
    ap.add_argument("--workload", type=int, default=1, help="index into the benchmark configurations (default 1: the headline one)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--shape", type=str, default=None,
                    help="cell,T,B,NH,D[,fwd]: bf16 workload with the paper's recipe (Wx, dH ~ N(0,1), R ~ N(0,1/D), forget bias 3), "
                         "drawn on the GPU; no oracle timing")
    ap.add_argument("--sweep", action="store_true", help="run the paper's head-size / batch / sequence-length sweeps and print a table")
    ap.add_argument("--sweep-out", type=str, default=None, help="also write the sweep table to this file")
    ap.add_argument("--recompute", action="store_true",
                    help="backward pass without saved values (flashrnn_bwd_recompute): forward without a gate cache, the values formed again window by window")
    ap.add_argument("--trace-phases", action="store_true",
                    help="load the trace build of the library and print the mean clocks per time step and phase of the persistent kernels")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run only a plain elementwise copy of 256 MiB (reads 256 MiB, writes 256 MiB) five times and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (the time loop never crosses GPUs); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    if args.trace_phases:
        os.environ["FLASHRNN_LIB"] = "trace"
    import numpy as np
    import torch
    from paper_2412_07752_amd import api, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    if args.copy_calibration:
        n = 64 * 1024 * 1024
        src = torch.ones(n, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": True, "bytes_read": 4 * n, "bytes_written": 4 * n, "launches": 5}))
        return
    if args.sweep:
        sweep(args, torch, api, synth)
        return

    def dev(a, dt):
        if a is None:
            return None
        if dt == "bf16":
            return torch.from_numpy(synth.bf16_bits(a).view(np.int16)).cuda().view(torch.bfloat16)
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()

    if args.shape:
        f = args.shape.split(",")
        cell = {v: k for k, v in synth.CELL_NAMES.items()}[f[0]]
        w, tensors = draw_on_device(torch, synth, cell, int(f[1]), int(f[2]), int(f[3]), int(f[4]), len(f) < 6 or f[5] != "fwd", "sweep_" + "_".join(f))
        args.no_cpu_baseline = True
        inp = None
    else:
        w = synth.CONFIGS[args.workload]
        inp = synth.make_inputs(w)
        tensors = (dev(inp["Wx"], w.dtype), dev(inp["R"], w.dtype), dev(inp["b"], w.dtype), dev(inp["states0"], "f32"), dev(inp["dH"], w.dtype))
    bf16 = w.dtype == "bf16"
    T, B, NH, D, G, S = w.T, w.B, w.NH, w.D, w.G, w.S
    runner = Runner(w, tensors, api, torch, recompute=args.recompute)
    desc = runner.desc
    ms_per_step, fwd_ms, bwd_ms, launches = runner.run(args.steps, args.warmup)
    value = B * T / (ms_per_step * 1e-3)
    if args.trace_phases:
        names = {False: ["prefetch_issue", "barrier_rows_read", "wait_exchange_and_lds_fill", "barrier_rows_ready", "lds_reads_mfma_slice_sums",
                         "pointwise_publish", "stores_and_input_wait", "poll_first_round_trip"],
                 True: ["loads_pointwise_publish_dwx", "barrier_rows_read", "wait_exchange_and_lds_fill", "barrier_rows_ready",
                        "lds_reads_mfma_slice_sums", "input_wait", "-", "poll_first_round_trip"]}
        res = {"workload": w.name, "plan_signature": plan_signature(api, desc, w.backward), "unit": "shader clocks per time step, mean over waves",
               "fwd_kernel_ms": round(fwd_ms, 4), "bwd_kernel_ms": round(bwd_ms, 4)}
        for bwd in ([False, True] if w.backward else [False]):
            clocks, waves = api.flashrnn_trace_phases(desc, runner.ws, bwd)
            pc = plan_call(bwd, w.backward)
            groups_per_wg = max(1, -(-(NH * -(-B // api.flashrnn_plan_kernel(desc, pc)[1])) // max(1, api.flashrnn_plan(desc, pc)[0] // api.flashrnn_plan_kernel(desc, pc)[2])))
            per = {n: round(c / (T * groups_per_wg), 1) for n, c in zip(names[bwd], clocks) if n != "-"}
            per["sum"] = round(sum(per.values()), 1)
            per["waves_recorded"] = waves
            res["bwd" if bwd else "fwd"] = per
        print(json.dumps(res))
        return

    # ---- rooflines of the two persistent time-loop kernels
    H = NH * D
    esz = 2 if bf16 else 4
    flops_launch = 2.0 * G * D * H * B * T          # recurrent product (forward) / its transpose (backward), per launch
    peak = PEAK_BF16_MFMA_TFLOPS if bf16 else PEAK_F32_MFMA_TFLOPS
    sig = plan_signature(api, desc, w.backward)
    counters = {}
    cf = os.path.join(ROOT, "profiles", f"counters_{w.name}.txt")
    if os.path.exists(cf):
        for ln in open(cf):
            if ":" in ln and not ln.startswith("#"):
                k, v = ln.split(":", 1)
                counters[k.strip()] = v.strip()
    same_plan = counters.get("plan_signature") == sig
    source = {"file": os.path.relpath(cf, ROOT), "commit": counters.get("source_commit")} if same_plan else None
    kernels = {}
    for name, bwd, ms in (("fwd", False, fwd_ms), ("bwd", True, bwd_ms)):
        if bwd and not w.backward:
            continue
        wgs, per_head, waves = api.flashrnn_plan(desc, plan_call(bwd, w.backward))
        staged, bt, split = api.flashrnn_plan_kernel(desc, plan_call(bwd, w.backward))
        nbytes = algorithmic_bytes(w, esz, bwd, w.backward)
        tfl = flops_launch / (ms * 1e-3) / 1e12 if ms > 0 else 0.0
        gbs = nbytes / (ms * 1e-3) / 1e9 if ms > 0 else 0.0
        occ = min(wgs, DEVICE_CUS)
        kernels[name] = {
            "launch_ms": round(ms, 5), "us_per_time_step": round(ms * 1e3 / max(T, 1), 4), "workgroups": wgs, "occupied_cus": occ,
            "batch_tile_rows": bt, "staged_kernel": staged, "workgroups_per_group": split,
            "flops_per_launch": flops_launch, "mfma_TFLOPs": round(tfl, 3), "mfma_peak_TFLOPs": peak,
            "mfma_frac_whole_device": tfl / peak,
            "mfma_peak_of_occupied_cus_TFLOPs": peak * occ / DEVICE_CUS, "useful_mfma_frac_of_occupied_cus": tfl / (peak * occ / DEVICE_CUS),
            "algorithmic_bytes_per_launch": nbytes, "hbm_GBs": round(gbs, 2), "hbm_peak_GBs": PEAK_HBM_GBS, "hbm_frac": gbs / PEAK_HBM_GBS,
            "measured_hbm_bytes_per_launch": float(counters[f"{name}_bytes_per_launch"]) if same_plan and f"{name}_bytes_per_launch" in counters else None,
            "mfma_pipe_busy_share": float(counters[f"{name}_mfma_pipe_busy_share"]) if same_plan and f"{name}_mfma_pipe_busy_share" in counters else None,
        }
    dom = "bwd" if (w.backward and bwd_ms >= fwd_ms) else "fwd"
    k = kernels[dom]
    intensity = flops_launch / k["algorithmic_bytes_per_launch"]
    ridge = peak * 1e12 / (PEAK_HBM_GBS * 1e9)
    if intensity < ridge:
        roofline = {"bound": "hbm", "achieved": k["hbm_GBs"], "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": k["hbm_frac"]}
    else:
        roofline = {"bound": "mfma", "achieved": k["mfma_TFLOPs"], "peak": peak, "unit": "TFLOP/s", "frac": k["mfma_frac_whole_device"]}
    roofline.update({
        "traffic": k["measured_hbm_bytes_per_launch"], "traffic_source": source,
        "kernel": ("backward" if dom == "bwd" else "forward") + " time-loop kernel", "launch_ms": k["launch_ms"], "launches_timed": launches,
        "algorithmic_bytes_per_launch": k["algorithmic_bytes_per_launch"], "arithmetic_intensity_flop_per_byte": round(intensity, 2),
        "ridge_flop_per_byte": round(ridge, 1), "plan_signature": sig, "kernels": kernels,
    })

    cpu = None
    if not args.no_cpu_baseline:
        import oracle  # the fp64 oracle as it stands, timed on this machine's host cores
        # bounded sample: the first Tc time steps of the same inputs (runtime is linear in T, paper App. H.3)
        work_per_step = (3 if w.backward else 1) * 2.0 * G * D * H * B
        Tc = max(1, min(T, int(40e9 / work_per_step)))
        f64 = lambda a: None if a is None else np.ascontiguousarray(a, dtype=np.float64)
        oWx, oR, ob, os0 = f64(inp["Wx"][:Tc]), f64(inp["R"]), f64(inp["b"]), f64(inp["states0"])
        odH = f64(inp["dH"][:Tc]) if w.backward else None
        reps, c0 = 0, time.perf_counter()
        while True:   # whole passes over the sample until a few seconds of wall clock are spent
            st = oracle.fwd(w.cell, oWx, oR, ob, os0)
            if w.backward:
                oracle.bwd(w.cell, oWx, oR, ob, st, odH)
            reps += 1
            c1 = time.perf_counter()
            if c1 - c0 >= 5.0 or reps >= 100:
                break
        cpu = {"value": reps * B * Tc / (c1 - c0), "unit": "B*T steps/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": f"first {Tc} of {T} time steps of the same inputs, all {B} rows and {NH} heads, "
                         f"{'fwd+bwd' if w.backward else 'fwd'}, fp64, {reps} passes in {c1 - c0:.2f} s"}

    line = {
        "metric": "fwd+bwd B*T steps/sec per RNN layer (sLSTM); recurrent-GEMM MFMA utilisation" if (args.workload == 1 and not args.shape)
                  else "B*T steps/sec per RNN layer",
        "value": value, "unit": "B*T steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
        "config": {"workload": w.name, "cell": synth.CELL_NAMES[w.cell], "B": B, "T": T, "NH": NH, "D": D,
                   "pass": ("fwd+bwd (values for the backward pass formed again, none saved)" if (args.recompute and w.backward) else
                            "fwd+bwd" if w.backward else "fwd"), "states_dtype": "f32"},
        "roofline": roofline, "cpu_baseline": cpu,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
