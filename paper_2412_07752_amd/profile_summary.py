"""Turns the rocprofv3 output of one workload into the text summary kept under profiles/ (counters_<workload>.txt).

Runs on the GPU machine after the profiling runs (it asks the library for the launch plan, which depends on the device);
it launches nothing itself.  The runs it expects under --dir, each made from /tmp with TMPDIR=/tmp and with
B = `python3 bench.py --workload <i> --no-cpu-baseline`:

    kt/            rocprofv3 --kernel-trace --stats --output-format csv -d <dir>/kt -o kt -- B --steps <K> --warmup <W>
    FETCH_SIZE/    rocprofv3 --pmc FETCH_SIZE --output-format csv -d <dir>/FETCH_SIZE -o p -- B --steps 3 --warmup 1
    WRITE_SIZE/    rocprofv3 --pmc WRITE_SIZE ...                                       (same command, other counter)
    copy_FETCH_SIZE/, copy_WRITE_SIZE/   the same two counters over `python3 bench.py --copy-calibration`
    sq_a/          rocprofv3 --pmc SQ_BUSY_CU_CYCLES SQ_WAVE_CYCLES SQ_ACTIVE_INST_VALU SQ_ACTIVE_INST_LDS SQ_ACTIVE_INST_VMEM
                       SQ_VALU_MFMA_BUSY_CYCLES SQ_WAIT_INST_ANY SQ_WAIT_INST_LDS ... -- B --steps 3 --warmup 1
    sq_b/          rocprofv3 --pmc SQ_INSTS_VALU SQ_INSTS_MFMA SQ_INSTS_LDS SQ_INSTS_VMEM_RD SQ_INSTS_VMEM_WR SQ_WAIT_ANY
                       SQ_LDS_IDX_ACTIVE SQ_LDS_BANK_CONFLICT ... -- B --steps 3 --warmup 1

    python3 -m paper_2412_07752_amd.profile_summary --workload <i> --dir <dir> --commit <git commit of the tree> --out <file>

Any of the counter runs may be missing; its lines are then left out.  FETCH_SIZE / WRITE_SIZE are KiB per dispatch and
are scaled by what the same counter reads for the copy kernel of known size (five copies of 256 MiB after one fill).
"""
import argparse
import collections
import csv
import glob
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

# (the packing kernels are called pack_r_fwd_kernel / pack_r_bwd_kernel: they are looked for first)
KINDS = (("pack_r", ("pack_r",)), ("sum_slices", ("sum_slices",)), ("dr_gemm", ("dr_gemm",)),
         ("fwd", ("fwd_tile_kernel", "fwd_kernel")), ("bwd", ("bwd_tile_kernel", "bwd_kernel")))


def kind_of(kernel_name):
    for kind, tags in KINDS:
        if any(t in kernel_name for t in tags):
            return kind
    return None


def counter_means(run_dir):
    """kind -> counter -> (mean per dispatch, dispatches); also the raw kernel name per kind."""
    files = glob.glob(os.path.join(run_dir, "**", "*counter_collection.csv"), recursive=True)
    if not files:
        return None, {}
    acc = collections.defaultdict(lambda: collections.defaultdict(list))
    names = {}
    for r in csv.DictReader(open(files[0])):
        k = kind_of(r["Kernel_Name"]) or ("copy" if "elementwise" in r["Kernel_Name"] else None)
        if k:
            acc[k][r["Counter_Name"]].append(float(r["Counter_Value"]))
            names[k] = r["Kernel_Name"]
    return {k: {c: (sum(v) / len(v), len(v)) for c, v in d.items()} for k, d in acc.items()}, names


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", type=int, required=True)
    ap.add_argument("--dir", required=True)
    ap.add_argument("--commit", default="unknown")
    ap.add_argument("--out", required=True)
    ap.add_argument("--kt-steps", default="K")
    a = ap.parse_args()

    import bench
    from paper_2412_07752_amd import api, synth
    w = synth.CONFIGS[a.workload]
    bf16 = w.dtype == "bf16"
    esz = 2 if bf16 else 4
    desc = api.make_desc(w.cell, w.T, w.B, w.NH, w.D, api.FLASHRNN_BF16 if bf16 else api.FLASHRNN_F32)
    sig = bench.plan_signature(api, desc, w.backward)
    B = f"python3 bench.py --workload {a.workload} --no-cpu-baseline"
    out = [f"# rocprofv3 summary of workload {w.name} ({synth.CELL_NAMES[w.cell]}, {'fwd+bwd' if w.backward else 'fwd'}, {w.dtype} I/O, "
           f"B={w.B} T={w.T} NH={w.NH} D={w.D})",
           "# every run from /tmp with TMPDIR=/tmp; B = " + B,
           f"source_commit: {a.commit}",
           f"plan_signature: {sig}"]
    flops = 2.0 * w.G * w.D * w.NH * w.D * w.B * w.T
    out.append(f"recurrent_flops_per_launch: {flops:.0f}")
    for kind, bwd in (("fwd", False), ("bwd", True)):
        if bwd and not w.backward:
            continue
        out.append(f"{kind}_algorithmic_bytes_per_launch: {bench.algorithmic_bytes(w, esz, bwd, w.backward)}")

    # ---- kernel trace
    ks = glob.glob(os.path.join(a.dir, "kt", "**", "*kernel_stats.csv"), recursive=True)
    avg_ns = {}
    if ks:
        out.append(f"# kernel durations: rocprofv3 --kernel-trace --stats --output-format csv -d <dir>/kt -o kt -- B --steps {a.kt_steps} (ns)")
        for r in csv.DictReader(open(ks[0])):
            out.append(f"#   {r['Name'][:110]} | calls {r['Calls']} | avg {float(r['AverageNs']):.0f} | min {r['MinNs']} | max {r['MaxNs']}")
            k = kind_of(r["Name"])
            if k:
                avg_ns[k] = float(r["AverageNs"])
        for k, v in avg_ns.items():
            out.append(f"{k}_avg_ns: {v:.0f}")

    # ---- HBM traffic
    fe, names = counter_means(os.path.join(a.dir, "FETCH_SIZE"))
    wr, _ = counter_means(os.path.join(a.dir, "WRITE_SIZE"))
    cfe, _ = counter_means(os.path.join(a.dir, "copy_FETCH_SIZE"))
    cwr, _ = counter_means(os.path.join(a.dir, "copy_WRITE_SIZE"))
    if fe and wr and cfe and cwr and "copy" in cfe and "copy" in cwr:
        kib = 262144.0
        m, n = cfe["copy"]["FETCH_SIZE"]
        f_scale = kib / (m * n / 5.0)       # n dispatches of the elementwise kernel: one fill (reads nothing) and five copies
        w_scale = kib / cwr["copy"]["WRITE_SIZE"][0]
        out.append("# HBM traffic: rocprofv3 --pmc FETCH_SIZE (then WRITE_SIZE) --output-format csv -d <dir>/<counter> -o p -- B --steps 3 --warmup 1")
        out.append("#   calibration: the same over `python3 bench.py --copy-calibration` (one fill + five copies of 256 MiB)")
        out.append(f"copy_scale_FETCH_SIZE: {f_scale:.4f}")
        out.append(f"copy_scale_WRITE_SIZE: {w_scale:.4f}")
        for kind in ("fwd", "bwd", "dr_gemm"):
            if kind in fe and kind in wr:
                r_b = fe[kind]["FETCH_SIZE"][0] * f_scale * 1024
                w_b = wr[kind]["WRITE_SIZE"][0] * w_scale * 1024
                out.append(f"#   {kind}: {names.get(kind, '')[:100]}")
                out.append(f"{kind}_bytes_read_per_launch: {r_b:.0f}")
                out.append(f"{kind}_bytes_written_per_launch: {w_b:.0f}")
                out.append(f"{kind}_bytes_per_launch: {r_b + w_b:.0f}")

    # ---- SQ counters
    sq = {}
    for run in ("sq_a", "sq_b"):
        m, _ = counter_means(os.path.join(a.dir, run))
        for k, d in (m or {}).items():
            sq.setdefault(k, {}).update({c: v[0] for c, v in d.items()})
    if sq:
        out.append("# SQ counters (means per dispatch; SQ_WAVE_CYCLES, SQ_BUSY_CU_CYCLES and the SQ_ACTIVE_* / SQ_WAIT_* counters tick once per 4 clocks):")
        out.append("#   rocprofv3 --pmc SQ_BUSY_CU_CYCLES SQ_WAVE_CYCLES SQ_ACTIVE_INST_VALU SQ_ACTIVE_INST_LDS SQ_ACTIVE_INST_VMEM SQ_VALU_MFMA_BUSY_CYCLES "
                   "SQ_WAIT_INST_ANY SQ_WAIT_INST_LDS --output-format csv -d <dir>/sq_a -o p -- B --steps 3 --warmup 1")
        out.append("#   rocprofv3 --pmc SQ_INSTS_VALU SQ_INSTS_MFMA SQ_INSTS_LDS SQ_INSTS_VMEM_RD SQ_INSTS_VMEM_WR SQ_WAIT_ANY SQ_LDS_IDX_ACTIVE "
                   "SQ_LDS_BANK_CONFLICT --output-format csv -d <dir>/sq_b -o p -- B --steps 3 --warmup 1")
        for kind in ("fwd", "bwd", "dr_gemm"):
            if kind not in sq:
                continue
            m = sq[kind]
            out.append(f"#   {kind}: " + ", ".join(f"{c} {m[c]:.0f}" for c in sorted(m)))
            if kind == "dr_gemm":
                if "SQ_INSTS_VALU" in m and m.get("SQ_INSTS_MFMA"):
                    out.append(f"dr_gemm_valu_per_mfma_instruction: {m['SQ_INSTS_VALU'] / m['SQ_INSTS_MFMA']:.2f}")
                continue
            wgs, _, waves = api.flashrnn_plan(desc, bench.plan_call(kind == "bwd", w.backward))
            nw, simds = wgs * waves, wgs * min(4, waves)
            if "SQ_WAVE_CYCLES" in m:
                clocks = m["SQ_WAVE_CYCLES"] * 4 / nw      # mean lifetime of a wave in clocks
                out.append(f"{kind}_kernel_clocks: {clocks:.0f}")
                out.append(f"{kind}_clocks_per_time_step: {clocks / max(w.T, 1):.0f}")
                if "SQ_VALU_MFMA_BUSY_CYCLES" in m:
                    out.append(f"{kind}_mfma_busy_clocks_per_simd_and_time_step: {m['SQ_VALU_MFMA_BUSY_CYCLES'] / simds / max(w.T, 1):.0f}")
                    out.append(f"{kind}_mfma_pipe_busy_share: {m['SQ_VALU_MFMA_BUSY_CYCLES'] / simds / clocks:.4f}")
                if "SQ_WAIT_INST_ANY" in m:
                    out.append(f"{kind}_wave_time_waiting_for_an_instruction_share: {m['SQ_WAIT_INST_ANY'] / m['SQ_WAVE_CYCLES']:.4f}")
                if "SQ_WAIT_INST_LDS" in m:
                    out.append(f"{kind}_wave_time_waiting_for_lds_share: {m['SQ_WAIT_INST_LDS'] / m['SQ_WAVE_CYCLES']:.4f}")
                if "SQ_WAIT_ANY" in m:
                    out.append(f"{kind}_wave_time_stalled_share: {m['SQ_WAIT_ANY'] / m['SQ_WAVE_CYCLES']:.4f}   # any wait: barrier, waitcnt, sleep")
            if "SQ_LDS_BANK_CONFLICT" in m and m.get("SQ_LDS_IDX_ACTIVE"):
                out.append(f"{kind}_lds_bank_conflict_share_of_lds_active_cycles: {m['SQ_LDS_BANK_CONFLICT'] / m['SQ_LDS_IDX_ACTIVE']:.4f}")
            if "SQ_INSTS_VALU" in m:
                out.append(f"{kind}_valu_instructions_per_wave_and_time_step: {m['SQ_INSTS_VALU'] / nw / max(w.T, 1):.1f}")
            if "SQ_INSTS_MFMA" in m:
                out.append(f"{kind}_mfma_instructions_per_wave_and_time_step: {m['SQ_INSTS_MFMA'] / nw / max(w.T, 1):.1f}")
            if "SQ_INSTS_LDS" in m:
                out.append(f"{kind}_lds_instructions_per_wave_and_time_step: {m['SQ_INSTS_LDS'] / nw / max(w.T, 1):.1f}")

    # ---- fractions a reader can recompute from the lines above (peaks: 2500 TFLOP/s dense bf16, 157.3 f32, 8000 GB/s)
    peak = 2500.0 if bf16 else 157.3
    for kind, bwd in (("fwd", False), ("bwd", True)):
        if kind not in avg_ns:
            continue
        s = avg_ns[kind] * 1e-9
        wgs = api.flashrnn_plan(desc, bench.plan_call(bwd, w.backward))[0]
        nb = bench.algorithmic_bytes(w, esz, bwd, w.backward)
        out.append(f"{kind}_mfma_frac_whole_device: {flops / s / 1e12 / peak:.5f}")
        out.append(f"{kind}_useful_mfma_frac_of_occupied_cus: {flops / s / 1e12 / (peak * min(wgs, 256) / 256):.5f}   # {min(wgs, 256)} CUs")
        out.append(f"{kind}_hbm_frac_algorithmic_bytes: {nb / s / 1e9 / 8000.0:.5f}")
    os.makedirs(os.path.dirname(os.path.abspath(a.out)), exist_ok=True)
    open(a.out, "w").write("\n".join(out) + "\n")
    print("\n".join(out))


if __name__ == "__main__":
    main()
