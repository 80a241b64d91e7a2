"""Writes tests/golden/bf16_floor.txt: what bf16 STORAGE alone costs on the named bf16 workloads.

For each workload and conditioning std the script runs ONE image-only patch call (last patch) of the CPU oracle at
the configured size and depth on the seeded synthetic stale K/V buffer, twice: exactly (float64), and with the
oracle's storage-rounding probe set to round-to-nearest-even bf16 (every tensor a bf16 implementation keeps in bf16
between two contractions is rounded; all arithmetic stays float64).  The stored number is
max|y_rounded - y_exact| / rms(y_exact): the error that NO implementation with bf16 operands can avoid on that
input, in the metric of the parity bar.  Only oracle/ and the input generators are used; nothing here touches the
HIP library.  Several minutes of CPU per line (the big workloads are Tflops of float64 work).

    python tests/golden/make_bf16_floor.py [C2 C3 C4 C5] [--std 0.5 1.0]
"""
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
sys.path.insert(0, ROOT)

import workloads as wl  # noqa: E402
from oracle.pf_oracle import StageOracle  # noqa: E402


def floor_of_last_patch(cfg):
    W, A = wl.make_weights(cfg), wl.make_activations(cfg)
    n, p = wl.patch_rows(cfg), cfg["n_patches"] - 1
    xp = A["x"][p * n:(p + 1) * n]
    exact = StageOracle(cfg, W)
    ys = []
    for probe in (None, wl.round_to_bf16):
        orc = exact if probe is None else StageOracle(cfg, exact.layers, storage_round=probe)
        orc.kv_init(None, text=A["text"] if cfg["kind"] == 1 else None)
        for l in range(cfg["n_layers"]):
            k, v = wl.make_kv_fill(cfg, l)
            orc.set_kv(l, k, v)
        ys.append(orc.patch_forward(xp, A["cond"], p))
        orc.kbuf, orc.vbuf = [], []          # free the buffers before the next run
    ref, got = ys
    rms = float(np.sqrt(np.mean(ref ** 2)))
    return float(np.max(np.abs(got - ref))) / rms, float(np.sqrt(np.mean((got - ref) ** 2))) / rms, rms


def main():
    args = sys.argv[1:]
    stds = (0.5, 1.0)
    if "--std" in args:
        i = args.index("--std")
        stds = tuple(float(a) for a in args[i + 1:])
        args = args[:i]
    names = args or ["C2", "C3", "C4", "C5"]
    path = os.path.join(HERE, "bf16_floor.txt")
    old = {}
    if os.path.exists(path):
        for line in open(path):
            f = line.split()
            if len(f) >= 5 and not line.startswith("#"):
                old[(f[0], float(f[1]))] = line.rstrip("\n")
    for name in names:
        for std in stds:
            cfg = wl.variant(wl.CONFIGS[name], cond_std=std)
            t0 = time.time()
            mx, rel, rms = floor_of_last_patch(cfg)
            old[(name, std)] = f"{name} {std} {mx:.4e} {rel:.4e} {rms:.4f}"
            print(old[(name, std)], f"({time.time() - t0:.0f} s)", flush=True)
            with open(path, "w") as fh:
                fh.write("# bf16 storage floor of one image-only patch call (last patch) at full size and depth on the synthetic\n"
                         "# stale buffer; written by tests/golden/make_bf16_floor.py from the CPU oracle alone.\n"
                         "# workload  cond_std  max|err|/rms  rms(err)/rms  rms(y)\n")
                for k in sorted(old):
                    fh.write(old[k] + "\n")


if __name__ == "__main__":
    main()
