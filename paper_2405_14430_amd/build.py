"""Build libpfstage.so (HIP kernels + C boundary) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libpfstage.so")
SOURCES = ["elementwise.hip", "gemm_simt.hip", "gemm_mfma.hip", "gemm_mfma_dl.hip", "attn_simt.hip", "attn_mfma.hip", "attn_mfma2.hip", "probe.hip", "tuning.hip", "stage.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         # packed-fp32 arithmetic is kept off for all device code
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


# Kernels that must not use scratch memory: their LDS fragment reads are asynchronous inline-assembly loads whose
# completion is tracked by hand, so a register spill between a read and its wait would save a value that has not
# arrived - wrong results, not just slow ones.  The compiler reports every kernel's scratch size; the build checks it.
NO_SCRATCH = {"attn_mfma2.hip": "attn_mfma2_kernel"}


def _check_no_scratch(src, log):
    want = NO_SCRATCH.get(src)
    if not want:
        return
    name, seen = None, 0
    for line in log.splitlines():
        if "Function Name:" in line:
            name = line.split("Function Name:")[1].split()[0]
        elif name and want in name and ("ScratchSize [bytes/lane]:" in line or "VGPRs Spill:" in line):
            seen += 1
            if int(line.split(":")[-1].split()[0]) != 0:
                raise RuntimeError(f"{src}: kernel {name} spills ({line.split('remark:')[-1].strip()}); "
                                   "its hand-tracked LDS reads are only correct without register spills")
    if seen == 0:
        raise RuntimeError(f"{src}: the compiler reported no resource usage for {want}; cannot check for spills")


def _compile(src, objdir=OBJ, extra=()):
    obj = os.path.join(objdir, src.replace(".hip", ".o"))
    check = ["-Rpass-analysis=kernel-resource-usage"] if src in NO_SCRATCH else []
    cmd = [HIPCC, *FLAGS, *extra, *check, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    log = r.stdout + r.stderr
    out = "\n".join(l for l in log.splitlines() if "packed-fp32-ops" not in l and "kernel-resource-usage" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{out}")
    if "-DPF_TUNING" in extra:   # the tuning build's timeline stamps cost registers: report, do not refuse
        try:
            _check_no_scratch(src, log)
        except RuntimeError as e:
            out += f"\nwarning (tuning build): {e}"
    else:
        _check_no_scratch(src, log)
    return obj, out


def build(verbose=False, out=LIB, tuning=False):
    """tuning=True: a -DPF_TUNING build (plan constants become variables behind pf_tune(); for sweeps on the GPU,
    written to `out`, which must then not be the shipped library's path)."""
    if tuning and os.path.abspath(out) == LIB:
        raise ValueError("a tuning build must not replace the shipped library")
    objdir = OBJ + ("_tuning" if tuning else "")
    extra = ("-DPF_TUNING",) if tuning else ()
    os.makedirs(objdir, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        results = list(ex.map(lambda src: _compile(src, objdir, extra), SOURCES))
    for _, log in results:
        if verbose and log.strip():
            print(log)
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out, *[o for o, _ in results]]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout + r.stderr)
    return out


if __name__ == "__main__":
    if "--tuning" in sys.argv:      # python build.py --tuning /path/to/libpfstage_tuning.so
        print(build(verbose="-v" in sys.argv, out=sys.argv[sys.argv.index("--tuning") + 1], tuning=True))
    else:
        print(build(verbose="-v" in sys.argv))
