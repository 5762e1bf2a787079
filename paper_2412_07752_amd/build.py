"""Build libflashrnn.so (HIP, gfx950) in-tree.  `python -m paper_2412_07752_amd.build [--force]`.

Every translation unit is compiled with hipcc for gfx950 only, with the packed-FP32 VALU
instructions disabled (compiler flag, device side).  Objects land in csrc/_build (git-ignored), the
library next to the Python binding.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
OUT = os.path.join(HERE, "libflashrnn.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# -amdgpu-mfma-vgpr-form: MFMA results go to ordinary VGPRs.  Left to itself the compiler puts the accumulators of kernels with
# few waves into AGPRs and copies every result out again (16 moves per time step in the small tile kernels), and the kernels that
# hold R in all 512 registers spill less with it.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-mllvm", "-amdgpu-mfma-vgpr-form", "-I", INCLUDE, "-I", CSRC]


def sources():
    return sorted(f for f in os.listdir(CSRC) if f.endswith(".hip"))


def _newest_header():
    hs = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")] + [os.path.join(INCLUDE, "flashrnn.h")]
    return max(os.path.getmtime(h) for h in hs)


def _compile(src, obj, extra=()):
    r = subprocess.run([HIPCC] + FLAGS + list(extra) + ["-c", os.path.join(CSRC, src), "-o", obj], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    log = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{log}")
    return log


def build(force=False, jobs=None, trace=False):
    """trace=True: the same sources with -DFLASHRNN_TRACE (per-phase clock stamps in the split-group kernels), as
    libflashrnn_trace.so; a measurement build, never what the tests or the benchmark's numbers run on."""
    bdir = os.path.join(CSRC, "_build_trace" if trace else "_build")
    flags_extra = ["-DFLASHRNN_TRACE"] if trace else []
    out = OUT.replace("libflashrnn.so", "libflashrnn_trace.so") if trace else OUT
    os.makedirs(bdir, exist_ok=True)
    hdr = _newest_header()
    todo, objs = [], []
    for src in sources():
        obj = os.path.join(bdir, src[:-4] + ".o")
        objs.append(obj)
        if force or not os.path.exists(obj) or os.path.getmtime(obj) < max(hdr, os.path.getmtime(os.path.join(CSRC, src))):
            todo.append((src, obj))
    jobs = jobs or min(8, os.cpu_count() or 1)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        for log in ex.map(lambda so: _compile(*so, extra=flags_extra), todo):
            if log.strip():
                print(log)
    if todo or not os.path.exists(out):
        subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", out])
    return out


if __name__ == "__main__":
    print(build(force="--force" in sys.argv, trace="--trace" in sys.argv))
