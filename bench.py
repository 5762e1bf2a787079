"""Benchmark of the FlashRNN hot path on one MI355X.

A "step" is one pass of the whole hot path -- flashrnn_fwd followed by flashrnn_bwd (time loop in
both directions, dR GEMM, db reduction) -- over one batch of synthetic input, by default the
configuration the headline metric is quoted on (sLSTM, B=16, T=256, NH=4, D=192, bf16 I/O with f32
states).  Inputs are resident in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload IDX] [--no-cpu-baseline]
    python bench.py --copy-calibration     # a plain copy of known size, for scaling rocprofv3's HBM counters
    python bench.py --shape slstm,1024,16,4,192   # any (cell, T, B, NH, D) of the paper's sweeps; add ",fwd" for forward only

roofline.traffic is the measured HBM traffic per launch of the dominant kernel, taken from the summary
of the two rocprofv3 --pmc runs under profiles/ (hbm_traffic_<workload>.txt) when that file is there;
roofline.mfma_busy_frac_of_occupied_cus likewise from sq_counters_<workload>.txt.  frac_of_occupied_cus
counts the useful flops only (4 of the 16 batch columns of an MFMA tile carry data with 4-row batch tiles).
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
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run only a plain elementwise copy of 256 MiB (reads 256 MiB, writes 256 MiB) five times and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (the time loop never crosses GPUs); use --gpus 1", file=sys.stderr)
        sys.exit(2)

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
    def dev(a, dt):
        if a is None:
            return None
        if dt == "bf16":
            return torch.from_numpy(synth.bf16_bits(a).view(np.int16)).cuda().view(torch.bfloat16)
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()

    if args.shape:
        f = args.shape.split(",")
        cell = {v: k for k, v in synth.CELL_NAMES.items()}[f[0]]
        w = synth.Workload("sweep_" + "_".join(f), cell, int(f[1]), int(f[2]), int(f[3]), int(f[4]), "bf16", len(f) < 6 or f[5] != "fwd")
        args.no_cpu_baseline = True
        gen = torch.Generator(device="cuda")
        gen.manual_seed(0)
        Wx = torch.randn((w.T, w.B, w.G, w.NH, w.D), device="cuda", generator=gen).bfloat16()
        R = (torch.randn((w.NH, w.D, w.G, w.D), device="cuda", generator=gen) / w.D ** 0.5).bfloat16()
        b = torch.zeros((w.NH, w.G, w.D), device="cuda")
        if cell != synth.CELL_GRU:
            b[:, synth.FORGET_GATE] = 3.0
        b = b.bfloat16()
        s0 = None
        dH = torch.randn((w.T, w.B, w.NH, w.D), device="cuda", generator=gen).bfloat16() if w.backward else None
        inp = None
    else:
        w = synth.CONFIGS[args.workload]
        inp = synth.make_inputs(w)
        Wx, R, b = dev(inp["Wx"], w.dtype), dev(inp["R"], w.dtype), dev(inp["b"], w.dtype)
        s0 = dev(inp["states0"], "f32")
        dH = dev(inp["dH"], w.dtype)
    bf16 = w.dtype == "bf16"
    T, B, NH, D, G, S = w.T, w.B, w.NH, w.D, w.G, w.S
    desc = api.make_desc(w.cell, T, B, NH, D, api.FLASHRNN_BF16 if bf16 else api.FLASHRNN_F32)
    ws = api.alloc_workspace(desc, "cuda")
    states = torch.empty((T + 1, S, B, NH, D), dtype=torch.float32, device="cuda")
    cache = torch.empty(max(api.flashrnn_gate_cache_bytes(desc), 16), dtype=torch.uint8, device="cuda") if w.backward else None
    io_dt = torch.bfloat16 if bf16 else torch.float32
    out = None
    if w.backward:
        out = (torch.empty((T, B, G, NH, D), dtype=io_dt, device="cuda"), torch.empty((NH, D, G, D), dtype=torch.float32, device="cuda"),
               torch.empty((NH, G, D), dtype=torch.float32, device="cuda"), torch.empty((S, B, NH, D), dtype=torch.float32, device="cuda"))

    def step():
        api.flashrnn_fwd(w.cell, Wx, R, b, s0, save_for_backward=w.backward, workspace=ws, states=states, gate_cache=cache)
        if w.backward:
            api.flashrnn_bwd(w.cell, R, b, states, cache, dH, None, workspace=ws, out=out)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    api.flashrnn_check(desc, ws)
    api.flashrnn_profile_enable(True)   # HIP events around the persistent kernels, on the launch stream
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    fwd_ms, nf = api.flashrnn_profile_kernel_ms(False)
    bwd_ms, nb = api.flashrnn_profile_kernel_ms(True) if w.backward else (0.0, 0)
    api.flashrnn_profile_enable(False)
    api.flashrnn_check(desc, ws)
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = B * T / (ms_per_step * 1e-3)

    # ---- roofline of the dominant kernel: the longer of the two persistent time-loop kernels.
    # Algorithmic work per (b, t): forward 2*G*D*H flops of recurrent product; backward the same for dh.
    H = NH * D
    flops_launch = 2.0 * G * D * H * B * T
    dom_bwd = w.backward and bwd_ms >= fwd_ms
    dom_ms = bwd_ms if dom_bwd else fwd_ms
    peak = PEAK_BF16_MFMA_TFLOPS if bf16 else PEAK_F32_MFMA_TFLOPS
    achieved = flops_launch / (dom_ms * 1e-3) / 1e12 if dom_ms > 0 else 0.0
    wgs, per_head, waves = api.flashrnn_plan(desc, dom_bwd)
    staged, batch_tile, split = api.flashrnn_plan_kernel(desc, dom_bwd)
    esz = 2 if bf16 else 4
    nc = 5 if w.cell == synth.CELL_SLSTM else 4
    if dom_bwd:   # reads: saved values, states t and t-1 (what the cell needs), dH; writes dWx
        bytes_launch = B * T * H * (nc * esz + esz + G * esz) + B * T * H * 4 * (2 if w.cell != synth.CELL_GRU else 1) * (2 if w.cell == synth.CELL_SLSTM else 1)
    else:         # reads Wx; writes states and saved values
        bytes_launch = B * T * H * (G * esz + S * 4 + (nc * esz if w.backward else 0))
    traffic = None   # measured HBM bytes per launch of the dominant kernel (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled)
    tf = os.path.join(ROOT, "profiles", f"hbm_traffic_{w.name}.txt")
    if os.path.exists(tf):
        for ln in open(tf):
            key = "bwd_bytes_per_launch:" if dom_bwd else "fwd_bytes_per_launch:"
            if ln.startswith(key):
                traffic = float(ln.split(":")[1])
    busy = None      # measured share of the kernel's duration in which a SIMD's matrix pipe is busy (SQ_VALU_MFMA_BUSY_CYCLES)
    sf = os.path.join(ROOT, "profiles", f"sq_counters_{w.name}.txt")
    if os.path.exists(sf):
        for ln in open(sf):
            if ln.startswith("bwd_mfma_busy_frac:" if dom_bwd else "fwd_mfma_busy_frac:"):
                busy = float(ln.split(":")[1])
    roofline = {
        "bound": "mfma", "kernel": ("backward time-loop kernel" if dom_bwd else "forward time-loop kernel"), "achieved": round(achieved, 4), "peak": peak,
        "unit": "TFLOP/s", "frac": achieved / peak, "traffic": traffic,
        "launch_ms": round(dom_ms, 5), "launches_timed": nb if dom_bwd else nf,
        "flops_per_launch": flops_launch,
        "workgroups": wgs, "batch_tile_rows": batch_tile, "staged_kernel": staged, "workgroups_per_group": split,
        "frac_of_occupied_cus": achieved / (peak * wgs / DEVICE_CUS),
        "mfma_busy_frac_of_occupied_cus": busy,
        "hbm_stream_GBs": round(bytes_launch / (dom_ms * 1e-3) / 1e9, 2) if dom_ms > 0 else None,
        "hbm_frac": (bytes_launch / (dom_ms * 1e-3) / 1e9) / PEAK_HBM_GBS if dom_ms > 0 else None,
        "fwd_kernel_ms": round(fwd_ms, 5), "bwd_kernel_ms": round(bwd_ms, 5),
    }

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
            if c1 - c0 >= 2.0 or reps >= 50:
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
                   "pass": "fwd+bwd" if w.backward else "fwd", "states_dtype": "f32"},
        "roofline": roofline, "cpu_baseline": cpu,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
