"""Patch-stage benchmark: one step = one pf_stage_patch_forward call (all rows of the hot path) on one patch of
a synthetic workload, inputs resident in HBM.  Prints ONE JSON line (tokens/s, ms per step, roofline of the
dominant kernel, CPU-oracle baseline).

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C4] [--others C2 C3 C5] [--no-cpu]

The headline workload is the Flux-scale stage C4 (the largest of the named single-GPU workloads: 7 blocks, patches of
2048 tokens over 16896 K/V rows, image-only call); the other bf16 workloads are measured the same way in the same run
and reported under "others".  Steps run as a diffusion step runs them: patch p = step mod M, the first patch of a
step derives the modulation vectors from the timestep embedding, the other M - 1 reuse them (pf_cond.same_cond).
The K timed steps are one block; blocks are repeated until half a second of GPU time has been timed and the median
(and minimum) block is reported.  Only one GPU is used; --gpus N with N > 1 exits with a message.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import workloads as wl  # noqa: E402

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_F32_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0
MIN_TIMED_SECONDS = 0.5
MAX_BLOCKS = 200


def flops_per_launch(cfg, cls, rows):
    """Algorithmic flops of one launch of a kernel class on `rows` query/GEMM rows (2mnk per GEMM, 4 n Lkv d for
    attention's two contractions)."""
    d, F, Lkv = cfg["hidden"], cfg["mlp_dim"], wl.kv_rows(cfg)
    if cls == "attention":
        return 4.0 * rows * Lkv * d
    if cls == "xattn":
        return 4.0 * rows * cfg["text_len"] * d
    if cls == "gemm_qkv":
        return 2.0 * rows * 3 * d * d
    if cls in ("gemm_out", "gemm_xattn"):
        return 2.0 * rows * d * d
    if cls == "gemm_up":
        return 2.0 * rows * F * d
    if cls == "gemm_down":
        return 2.0 * rows * d * (F + (d if cfg["kind"] == 3 else 0))
    return 0.0


def call_flops(cfg, rows):
    """Algorithmic flops of one patch call on `rows` rows (image-only call: rows = n)."""
    d, F, Lkv, nl = cfg["hidden"], cfg["mlp_dim"], wl.kv_rows(cfg), cfg["n_layers"]
    per_tok = 2 * d * 3 * d + 4 * Lkv * d + 2 * d * d + 4 * d * F
    if cfg["kind"] == 1:
        per_tok += 4 * d * d + 4 * cfg["text_len"] * d
    return float(per_tok) * rows * nl


def bytes_per_launch(cfg, cls, rows):
    """Algorithmic HBM bytes of one launch of a streaming kernel class."""
    d = cfg["hidden"]
    esz = 2 if cfg["dtype"] == "bf16" else 4
    if cls == "ln_modulate":
        return rows * d * (4 + esz)           # fp32 residual row in, dtype row out
    if cls == "kv_scatter":
        return 2 * 2 * rows * d * esz         # k and v rows read and written once
    return 0


def _timed_blocks(run_block, steps):
    """Times blocks of exactly `steps` steps (device synchronised on both sides of each) until MIN_TIMED_SECONDS have
    been timed; returns the per-step milliseconds of every block."""
    import torch
    per_step, total = [], 0.0
    while total < MIN_TIMED_SECONDS and len(per_step) < MAX_BLOCKS:
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run_block()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        per_step.append(dt * 1e3 / steps)
        total += dt
    return per_step


def measure(name, steps, warmup, path=0):
    """Builds the stage of workload `name`, runs its real warm-up pass, and times patch calls.  Returns the result
    dictionary of the workload (timing, per-kernel-class figures, roofline of the dominant kernel)."""
    import torch
    from paper_2405_14430_amd import Stage

    cfg = wl.CONFIGS[name]
    n, M = wl.patch_rows(cfg), cfg["n_patches"]
    W, A = wl.make_weights(cfg), wl.make_activations(cfg)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    dt = torch.bfloat16 if cfg["dtype"] == "bf16" else torch.float32
    cond = dev(A["cond"])
    text = None
    if A["text"] is not None:
        text = dev(A["text"]).to(dt) if cfg["kind"] == 1 else dev(A["text"])
    st = Stage(cfg, W, kernel_path=path)
    del W
    st.kv_init(dev(A["x_prev"]), cond, text)
    x = dev(A["x"])
    xs = [x[p * n:(p + 1) * n].contiguous() for p in range(M)]
    ys = [torch.empty_like(t) for t in xs]
    torch.cuda.synchronize()

    def step(i, reuse=True):
        p = i % M
        st.patch_forward(xs[p], cond, p, out=ys[p], same_cond=reuse and p != 0)

    for i in range(warmup):
        step(i)
    blocks = _timed_blocks(lambda: [step(i) for i in range(steps)], steps)
    ms_per_step, ms_min = statistics.median(blocks), min(blocks)
    # the same with the modulation vectors derived in every call
    fresh = _timed_blocks(lambda: [step(i, reuse=False) for i in range(steps)], steps)
    flops = call_flops(cfg, n)
    res = {
        "workload": name, "ms_per_step": ms_per_step, "ms_per_step_min": ms_min, "blocks_timed": len(blocks),
        "steps_per_block": steps, "tokens_per_s": n / (ms_per_step * 1e-3),
        "tflops": flops / (ms_per_step * 1e-3) / 1e12, "ms_per_step_cond_derived_every_call": statistics.median(fresh),
        "patch_tokens": n, "flops_per_call": flops,
    }
    res["frac_of_bf16_mfma_peak"] = res["tflops"] / PEAK_BF16_TFLOPS

    # joint-attention kinds: the call that carries the text rows (patch 0 of a step) is heavier; time it too and give the
    # aggregate of a whole step's M calls (one with text, M - 1 without)
    if cfg["kind"] in (2, 3) and text is not None:
        tout = torch.empty_like(text)
        reps = max(4, min(steps, 40))
        for _ in range(2):
            st.patch_forward(xs[0], cond, 0, text=text, out=ys[0], text_out=tout)
        torch.cuda.synchronize()
        tt0 = time.perf_counter()
        for _ in range(reps):
            st.patch_forward(xs[0], cond, 0, text=text, out=ys[0], text_out=tout)
        torch.cuda.synchronize()
        ms_text = (time.perf_counter() - tt0) * 1e3 / reps
        step_ms = ms_text + (M - 1) * ms_per_step
        res["joint_step"] = {"ms_call_with_text_rows": ms_text, "text_rows": cfg["text_len"],
                             "ms_per_step_of_M_calls": step_ms, "tokens_per_s_over_step": M * n / (step_ms * 1e-3)}

    # second pass, same steps, with HIP events after every launch on the stage's stream
    st.profile(1)
    for i in range(steps):
        step(i)
    prof = st.profile_read()
    st.profile(0)
    # An event between two launches costs GPU time of its own.  The cost per launch is measured live: what the event
    # intervals of a step add up to, minus the step time of the pass without events, over the launches of a step.
    total_ms = sum(ms for ms, cnt in prof.values()) / steps
    total_launches = sum(cnt for ms, cnt in prof.values()) / steps
    event_overhead_us = max(0.0, (total_ms - ms_per_step) / max(total_launches, 1.0) * 1e3)
    kernels = {}
    for cls, (ms, cnt) in prof.items():
        if cnt:
            raw = ms / cnt * 1e3
            kernels[cls] = {"ms_per_step": (raw - event_overhead_us) * cnt / steps * 1e-3,
                            "launches_per_step": cnt / steps, "avg_us": raw - event_overhead_us,
                            "avg_us_with_event": raw}
    peak = PEAK_BF16_TFLOPS if cfg["dtype"] == "bf16" else PEAK_F32_TFLOPS
    for c in kernels:
        f = flops_per_launch(cfg, c, n)
        b = bytes_per_launch(cfg, c, n)
        if f:
            kernels[c]["tflops"] = f / (kernels[c]["avg_us"] * 1e-6) / 1e12
            kernels[c]["frac_of_peak"] = kernels[c]["tflops"] / peak
        if b:
            kernels[c]["gbs"] = b / (kernels[c]["avg_us"] * 1e-6) / 1e9
    # Group the launch classes by the kernel (symbol) that actually runs them - the unit rocprofv3 reports - and take
    # the group with the most time as the dominant kernel.
    d_, F_ = cfg["hidden"], cfg["mlp_dim"]
    gemm_shapes = {"gemm_qkv": (3 * d_, d_), "gemm_out": (d_, d_), "gemm_xattn": (d_, d_), "gemm_up": (F_, d_),
                   "gemm_down": (d_, F_ + (d_ if cfg["kind"] == 3 else 0))}
    dtc = 1 if cfg["dtype"] == "bf16" else 0
    groups = {}
    for c in kernels:
        f = flops_per_launch(cfg, c, n)
        if not f:
            continue
        if c in gemm_shapes:
            sym = st.lib.pf_gemm_kernel_name(dtc, path, n, gemm_shapes[c][0], gemm_shapes[c][1]).decode()
        else:
            sym = st.lib.pf_attention_kernel_name(dtc, path, cfg["head_dim"], n, 1 if c == "attention" else 0).decode()
        g = groups.setdefault(sym, {"ms": 0.0, "launches": 0.0, "flops": 0.0, "classes": []})
        g["ms"] += kernels[c]["ms_per_step"]
        g["launches"] += kernels[c]["launches_per_step"]
        g["flops"] += f * kernels[c]["launches_per_step"]
        g["classes"].append(c)
    dom = max(groups, key=lambda k: groups[k]["ms"])
    g = groups[dom]
    ach = g["flops"] / (g["ms"] * 1e-3) / 1e12
    # HBM-side bytes per launch of the dominant kernel: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this workload,
    # committed under profiles/ with the commit they were taken at (counters cannot be read from inside this process)
    traffic, traffic_src = None, None
    tpath = os.path.join(ROOT, "profiles", f"hbm_traffic_{name.lower()}.json")
    if os.path.exists(tpath):
        tj = json.load(open(tpath))
        t = tj.get("kernels", {}).get(dom)
        if t:
            traffic = t["fetch_bytes"] + t["write_bytes"]
            traffic_src = {"file": os.path.relpath(tpath, ROOT), "commit": tj.get("commit")}
    res["roofline"] = {"kernel": dom, "classes": g["classes"], "bound": "mfma" if cfg["dtype"] == "bf16" else "alu",
                       "achieved": ach, "peak": peak, "unit": "TFLOP/s", "frac": ach / peak, "traffic": traffic,
                       "traffic_source": traffic_src, "avg_launch_us": g["ms"] / g["launches"] * 1e3,
                       "launches_per_step": g["launches"], "flops_per_launch": g["flops"] / g["launches"],
                       "event_overhead_us": event_overhead_us}
    res["kernels"] = kernels
    # matrix work of the call (GEMMs + attention) against the peak: time spent in those launches only
    mm_ms = sum(k["ms_per_step"] for c, k in kernels.items() if flops_per_launch(cfg, c, n))
    res["matrix_kernels"] = {"ms_per_step": mm_ms, "tflops": flops / (mm_ms * 1e-3) / 1e12,
                             "frac_of_peak": flops / (mm_ms * 1e-3) / 1e12 / peak}
    st.destroy()
    del st, x, xs, ys
    torch.cuda.empty_cache()
    return res


def cpu_oracle_baseline(name):
    """The CPU oracle timed on this machine's host cores on a bounded sample of the workload: patch calls on synthetic stale
    K/V; for the workloads whose call is Tflops of float64 work, one call of a 2-layer cut of the stage (all layers
    have the same shape), scaled to the configured depth."""
    from oracle.pf_oracle import StageOracle
    cfg = wl.CONFIGS[name]
    n, M = wl.patch_rows(cfg), cfg["n_patches"]
    big = call_flops(cfg, n) > 1e12
    nl = 2 if big else cfg["n_layers"]
    cut = wl.variant(cfg, n_layers=nl)
    W, A = wl.make_weights(cut, n_layers=nl), wl.make_activations(cut)
    orc = StageOracle(cut, W)
    if cfg["kind"] == 1:
        orc.kv_init(None, text=A["text"])
    for l in range(nl):
        k, v = wl.make_kv_fill(cfg, l)
        orc.set_kv(l, k, v)
    calls, tc0 = 0, time.perf_counter()
    while True:
        p = (M - 1 - calls) % M
        orc.patch_forward(A["x"][p * n:(p + 1) * n], A["cond"], p)
        calls += 1
        if big or time.perf_counter() - tc0 > 10.0 or calls >= 8:
            break
    tc = time.perf_counter() - tc0
    try:
        from threadpoolctl import threadpool_info
        threads = max([i.get("num_threads", 1) for i in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count()
    scale = cfg["n_layers"] / nl
    sample = (f"{calls} patch_forward call(s) of {name} (n={n} tokens each, image only) on synthetic stale K/V, numpy "
              f"float64, {tc:.1f} s")
    if big:
        sample += f"; {nl} of the stage's {cfg['n_layers']} identical layers were run and the time scaled by {scale:g}"
    return {"value": calls * n / (tc * scale), "unit": "tokens/s", "cores": threads, "kind": "oracle", "sample": sample}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="C4")
    ap.add_argument("--others", nargs="*", default=None, help="further workloads measured in the same run "
                    "(default: the other named bf16 workloads)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--path", type=int, default=0, help="0 auto (MFMA for bf16), 1 force SIMT kernels")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the multi-GPU pipeline schedule is out of scope); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    others = args.others if args.others is not None else [w for w in ("C2", "C3", "C5") if w != args.workload]

    main_res = measure(args.workload, args.steps, args.warmup, args.path)
    cfg = wl.CONFIGS[args.workload]
    other_res = {}
    for w in others:
        r = measure(w, args.steps, args.warmup, args.path)
        other_res[w] = {k: r[k] for k in ("ms_per_step", "ms_per_step_min", "tokens_per_s", "tflops", "frac_of_bf16_mfma_peak",
                                          "ms_per_step_cond_derived_every_call", "patch_tokens", "matrix_kernels")}
        other_res[w]["roofline"] = {k: r["roofline"][k] for k in ("kernel", "classes", "achieved", "peak", "unit", "frac",
                                                                  "traffic", "avg_launch_us", "launches_per_step")}
        other_res[w]["kernel_avg_us"] = {c: round(k["avg_us"], 2) for c, k in r["kernels"].items()}
        if "joint_step" in r:
            other_res[w]["joint_step"] = r["joint_step"]

    # measured ceiling of the matrix pipes (register-only MFMA loop), beside the data-sheet peak
    mfma_loop = None
    if cfg["dtype"] == "bf16":
        from paper_2405_14430_amd import probe_mfma_tflops
        mfma_loop = probe_mfma_tflops()
    # measured device-to-device copy rate (256 MiB, read + write bytes), the yardstick for the streaming kernels' GB/s
    src_, dst_ = torch.empty(1 << 28, dtype=torch.uint8, device="cuda"), torch.empty(1 << 28, dtype=torch.uint8, device="cuda")
    dst_.copy_(src_)
    ce0, ce1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ce0.record()
    for _ in range(4):
        dst_.copy_(src_)
    ce1.record()
    ce1.synchronize()
    hbm_copy_gbs = 4 * 2 * (1 << 28) / (ce0.elapsed_time(ce1) * 1e-3) / 1e9
    del src_, dst_
    roofline = main_res["roofline"]
    roofline["mfma_loop_tflops"] = mfma_loop
    roofline["frac_of_mfma_loop"] = (roofline["achieved"] / mfma_loop) if mfma_loop else None

    cpu = None if args.no_cpu else cpu_oracle_baseline(args.workload)

    n, M = wl.patch_rows(cfg), cfg["n_patches"]
    out = {
        "metric": "patch-stage tokens/s", "value": main_res["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": main_res["ms_per_step"],
        "ms_per_step_min": main_res["ms_per_step_min"], "blocks_timed": main_res["blocks_timed"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": cfg["dtype"], "data": "synthetic",
        "config": {"workload": args.workload, "kind": cfg["kind"], "n_layers": cfg["n_layers"], "hidden": cfg["hidden"],
                   "heads": cfg["n_heads"], "head_dim": cfg["head_dim"], "mlp_dim": cfg["mlp_dim"],
                   "seq_img": cfg["seq_img"], "n_patches": M, "patch_tokens": n, "kv_rows": wl.kv_rows(cfg),
                   "text_len": cfg["text_len"], "call": "image-only patch call after a real warm-up pass; modulation "
                   "vectors derived on the first patch of a step and reused by the others"},
        "tflops": main_res["tflops"], "frac_of_bf16_mfma_peak": main_res["frac_of_bf16_mfma_peak"],
        "ms_per_step_cond_derived_every_call": main_res["ms_per_step_cond_derived_every_call"],
        "matrix_kernels": main_res["matrix_kernels"],
        "roofline": roofline, "cpu_baseline": cpu, "kernels": main_res["kernels"], "hbm_copy_gbs": hbm_copy_gbs,
        "others": other_res,
    }
    if "joint_step" in main_res:
        out["joint_step"] = main_res["joint_step"]
    print(json.dumps(out))


if __name__ == "__main__":
    main()
