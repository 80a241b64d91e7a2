"""Patch-number sweep (App. B ablation on M; Sec. 3.3 recommends M = N): for a workload at fixed sequence length, time the
stage's patch call for several patch counts M, and the full sampling-loop step (all M patches through N chained stages plus
the update) for one of them.  Prints one JSON line per measurement.

  python -m paper_2405_14430_amd.sweep --workload C2 --patches 2 4 8 16 32 [--stages 2] [--batch 1 2] [--iters 50]

On N devices one micro-step costs max over stages of (patch call + P2P); a smaller patch shortens the pipeline fill
(N - 1 micro-steps) but makes every operator smaller.  The sweep shows the second half on one device: tokens/s of the stage
as a function of M.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import workloads as wl  # noqa: E402  (seeded synthetic inputs; holds none of the method's arithmetic)


def call_flops(cfg, rows):
    """Algorithmic flops of one patch call on `rows` image rows."""
    d, F, Lkv, nl = cfg["hidden"], cfg["mlp_dim"], wl.kv_rows(cfg), cfg["n_layers"]
    per_tok = 2 * d * 3 * d + 4 * Lkv * d + 2 * d * d + 4 * d * F
    if cfg["kind"] == 1:
        per_tok += 4 * d * d + 4 * cfg["text_len"] * d
    return float(per_tok) * rows * nl


def _dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def _text(cfg, A):
    import torch
    if A["text"] is None:
        return None
    t = _dev(A["text"])
    return t.to(torch.bfloat16 if cfg["dtype"] == "bf16" else torch.float32) if cfg["kind"] == 1 else t


def sweep_patch_call(name, patches, iters, warmup):
    import torch
    from . import Stage
    base = wl.CONFIGS[name]
    W, A = wl.make_weights(base), wl.make_activations(base)
    cond, text, x = _dev(A["cond"]), _text(base, A), _dev(A["x"])
    xprev = _dev(A["x_prev"])
    for M in patches:
        if base["seq_img"] % M:
            continue
        cfg = wl.variant(base, n_patches=M)
        n = wl.patch_rows(cfg)
        st = Stage(cfg, W)
        st.kv_init(xprev, cond, text)
        xs = [x[p * n:(p + 1) * n] for p in range(M)]
        y = torch.empty_like(xs[0])
        calls = max(iters, M)
        for i in range(warmup):
            st.patch_forward(xs[i % M], cond, i % M, out=y)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(calls):
            st.patch_forward(xs[i % M], cond, i % M, out=y)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / calls
        print(json.dumps({"what": "patch_call", "workload": name, "n_patches": M, "patch_tokens": n,
                          "ms_per_call": ms, "ms_per_sweep_of_all_patches": ms * M,
                          "tokens_per_s": n / (ms * 1e-3), "tflops": call_flops(cfg, n) / (ms * 1e-3) / 1e12}),
              flush=True)
        st.destroy()
        del st


def sweep_batch(name, batches, iters, warmup):
    """Patch call of the workload at its own M for B images per call (B = 2: the conditional and unconditional image of
    classifier-free guidance share one call, Sec. 4.1 (CFG parallel) runs them on separate device groups instead)."""
    import torch
    from . import Stage
    base = wl.CONFIGS[name]
    W = wl.make_weights(base)
    M, n = base["n_patches"], wl.patch_rows(base)
    for B in batches:
        acts = [wl.make_activations(wl.variant(base, seed=base["seed"] + 100 * b)) for b in range(B)]
        stack = lambda k: _dev(np.stack([a[k] for a in acts], 0))
        cfg = dict(base, batch=B)
        cond, x, xprev = stack("cond"), stack("x"), stack("x_prev")
        text = None
        if acts[0]["text"] is not None:
            text = stack("text")
            if base["kind"] == 1:
                text = text.to(torch.bfloat16 if base["dtype"] == "bf16" else torch.float32)
        st = Stage(cfg, W)
        st.kv_init(xprev, cond, text)
        xs = [x[:, p * n:(p + 1) * n].contiguous() for p in range(M)]
        y = torch.empty_like(xs[0])
        for i in range(warmup):
            st.patch_forward(xs[i % M], cond, i % M, out=y)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(iters):
            st.patch_forward(xs[i % M], cond, i % M, out=y)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / iters
        print(json.dumps({"what": "batched_patch_call", "workload": name, "batch": B, "n_patches": M, "patch_tokens": n,
                          "ms_per_call": ms, "tokens_per_s": B * n / (ms * 1e-3),
                          "tflops": B * call_flops(base, n) / (ms * 1e-3) / 1e12}), flush=True)
        st.destroy()
        del st


def time_full_step(name, M, n_stages, steps):
    """One diffusion step after warm-up on one device: M patches x N stages + the update (the stages derive their
    modulation vectors on the first patch of the step and keep them for the others)."""
    import torch
    from .pipeline import Pipeline
    base = wl.variant(wl.CONFIGS[name], n_patches=M)
    W = wl.make_weights(base, n_layers=n_stages * base["n_layers"])
    A = wl.make_activations(base)
    conds, dts = wl.make_sampling(base, steps + 2)
    pipe = Pipeline(base, wl.split_stages(W, n_stages))
    text = _text(base, A)
    cd = [_dev(c) for c in conds]
    x = _dev(A["x"]).clone()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    pipe.run(x, cd[:1], dts[:1], warmup_steps=1, text=text)
    torch.cuda.synchronize()
    t_warm = (time.perf_counter() - t0) * 1e3
    x = pipe.run(x, cd[:2], dts[:2], warmup_steps=1, text=text)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    pipe.run(x, cd[2:], dts[2:], warmup_steps=0, text=text)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    L = base["seq_img"]
    fl = call_flops(base, L) * n_stages
    print(json.dumps({"what": "full_step", "workload": name, "n_patches": M, "stages": n_stages,
                      "layers": n_stages * base["n_layers"], "ms_per_step": ms, "ms_first_warmup_step": t_warm,
                      "tokens_per_s": L / (ms * 1e-3), "tflops": fl / (ms * 1e-3) / 1e12}), flush=True)
    pipe.destroy()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="C2")
    ap.add_argument("--patches", type=int, nargs="*", default=[2, 4, 8, 16, 32])
    ap.add_argument("--iters", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--stages", type=int, default=0, help="> 0: also time the full sampling-loop step with this many stages")
    ap.add_argument("--steps", type=int, default=4)
    ap.add_argument("--batch", type=int, nargs="*", default=[], help="also time the patch call for these images-per-call")
    args = ap.parse_args()
    import torch
    if not torch.cuda.is_available():
        print("sweep: no GPU visible", file=sys.stderr)
        sys.exit(1)
    sweep_patch_call(args.workload, args.patches, args.iters, args.warmup)
    if args.batch:
        sweep_batch(args.workload, args.batch, args.iters, args.warmup)
    if args.stages > 0:
        time_full_step(args.workload, wl.CONFIGS[args.workload]["n_patches"], args.stages, args.steps)


if __name__ == "__main__":
    main()
