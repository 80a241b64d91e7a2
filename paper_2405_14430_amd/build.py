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


def _compile(src, objdir=OBJ, extra=()):
    obj = os.path.join(objdir, src.replace(".hip", ".o"))
    cmd = [HIPCC, *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    out = "\n".join(l for l in (r.stdout + r.stderr).splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{out}")
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
