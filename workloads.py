"""Seeded synthetic inputs for the PipeFusion patch-stage workloads.

This module only *draws numbers*: configuration tables, Gaussian tensors of the
right shapes, and the bf16 storage rounding of those tensors.  It holds none of
the method's arithmetic and imports neither the CPU oracle nor the HIP binding;
both are fed from here so that they see bit-identical inputs.

The shapes stand in for the PixArt / SD3 / Flux.1 runs of the paper's
evaluation (Sec. 4, Experiments): trained weights and prompts are replaced by
Gaussians, and "the previous diffusion step's input" (Sec. 3.3, the stale
activations of timestep T+1) by x + 0.05*N(0,1).
"""
from __future__ import annotations

import numpy as np

# block kinds (must match include/pfstage.h)
KIND_ADALN_ZERO = 0          # classic DiT block, per-layer modulation Linear
KIND_ADALN_SINGLE_XATTN = 1  # PixArt: shared modulation + per-layer table, cross-attn to text
KIND_MMDIT_JOINT = 2         # SD3: two weight streams, one joint attention
KIND_SINGLE_STREAM = 3       # Flux single-stream: parallel attn+MLP, 2-D RoPE

_BASE = dict(text_len=0, cross_dim=0, ln_eps=1e-6, rope_theta=1e4, gelu_tanh=1,
             w_std=0.02, qk_gain=1.0, cond_std=None, qk_norm=0, joint_rope=0, txt_pre_only_last=0)


def _cfg(**kw):
    c = dict(_BASE)
    c.update(kw)
    if c["cond_std"] is None:
        c["cond_std"] = 1.0       # conditioning embedding N(0,1) unless the workload says otherwise (C4 does)
    assert c["hidden"] == c["n_heads"] * c["head_dim"]
    assert c["seq_img"] == c["grid_h"] * c["grid_w"]
    assert c["seq_img"] % c["n_patches"] == 0
    return c


CONFIGS = {
    # the five named workloads
    "C1": _cfg(kind=0, dtype="f32", n_layers=1, hidden=384, n_heads=6, head_dim=64, mlp_dim=1536,
               seq_img=256, grid_h=16, grid_w=16, n_patches=4, w_std="fan_in", seed=0),
    "C2": _cfg(kind=1, dtype="bf16", n_layers=4, hidden=1152, n_heads=16, head_dim=72, mlp_dim=4608,
               seq_img=4096, grid_h=64, grid_w=64, n_patches=8, text_len=120, cross_dim=1152, seed=1),
    # C3 and C5 draw the conditioning embedding at std 0.5, C4 at 0.25: the largest of {1, 0.5, 0.25} at which the bf16
    # STORAGE of the matrix operands alone (all arithmetic exact) costs at most two thirds of the 2e-2 parity bar on
    # the workload's own full-size call (tests/golden/bf16_floor.txt has the floors, tests/test_bf16_floor.py ties
    # these values to them).  On the 7-layer Flux-scale stage the format alone exceeds the bar at std 0.5 and 1: the
    # N(0,0.02) modulation weights at hidden 3072 turn a unit-variance embedding into gates of std 0.6.
    "C3": _cfg(kind=2, dtype="bf16", n_layers=3, hidden=1536, n_heads=24, head_dim=64, mlp_dim=6144,
               seq_img=4096, grid_h=64, grid_w=64, n_patches=8, text_len=154, seed=2, cond_std=0.5),
    "C4": _cfg(kind=3, dtype="bf16", n_layers=7, hidden=3072, n_heads=24, head_dim=128, mlp_dim=12288,
               seq_img=16384, grid_h=128, grid_w=128, n_patches=8, text_len=512, seed=3, cond_std=0.25),
    "C5": _cfg(kind=1, dtype="bf16", n_layers=4, hidden=1152, n_heads=16, head_dim=72, mlp_dim=4608,
               seq_img=65536, grid_h=256, grid_w=256, n_patches=16, text_len=120, cross_dim=1152, seed=4, cond_std=0.5),
    # structural twins: same block kinds and head sizes, small enough for a full
    # oracle sweep in seconds, with ragged row counts (text lengths and patch
    # sizes that are not multiples of any kernel tile).
    "C2s": _cfg(kind=1, dtype="bf16", n_layers=2, hidden=288, n_heads=4, head_dim=72, mlp_dim=1152,
                seq_img=1200, grid_h=30, grid_w=40, n_patches=4, text_len=37, cross_dim=160, seed=11),
    "C3s": _cfg(kind=2, dtype="bf16", n_layers=2, hidden=256, n_heads=4, head_dim=64, mlp_dim=1024,
                seq_img=1080, grid_h=30, grid_w=36, n_patches=4, text_len=77, seed=12),
    "C4s": _cfg(kind=3, dtype="bf16", n_layers=2, hidden=384, n_heads=3, head_dim=128, mlp_dim=1536,
                seq_img=1500, grid_h=30, grid_w=50, n_patches=5, text_len=45, seed=13),
    "C5s": _cfg(kind=1, dtype="bf16", n_layers=2, hidden=288, n_heads=4, head_dim=72, mlp_dim=1152,
                seq_img=4096, grid_h=64, grid_w=64, n_patches=16, text_len=120, cross_dim=288, seed=14),
    # fp32 twins of every kind (tight tolerance => wiring mistakes cannot hide in bf16 noise)
    "K0f": _cfg(kind=0, dtype="f32", n_layers=2, hidden=192, n_heads=3, head_dim=64, mlp_dim=512,
                seq_img=300, grid_h=15, grid_w=20, n_patches=3, w_std="fan_in", seed=20),
    "K1f": _cfg(kind=1, dtype="f32", n_layers=2, hidden=144, n_heads=2, head_dim=72, mlp_dim=384,
                seq_img=210, grid_h=14, grid_w=15, n_patches=3, text_len=19, cross_dim=96,
                w_std="fan_in", seed=21),
    "K2f": _cfg(kind=2, dtype="f32", n_layers=2, hidden=128, n_heads=2, head_dim=64, mlp_dim=320,
                seq_img=198, grid_h=11, grid_w=18, n_patches=3, text_len=29, w_std="fan_in", seed=22),
    "K3f": _cfg(kind=3, dtype="f32", n_layers=2, hidden=256, n_heads=2, head_dim=128, mlp_dim=640,
                seq_img=204, grid_h=12, grid_w=17, n_patches=3, text_len=21, w_std="fan_in", seed=23),
    # q / k RMSNorm (and RoPE on the two-stream joint block): the attention front end of the Flux-family blocks
    "K2n": _cfg(kind=2, dtype="f32", n_layers=2, hidden=128, n_heads=2, head_dim=64, mlp_dim=320,
                seq_img=198, grid_h=11, grid_w=18, n_patches=3, text_len=29, w_std="fan_in", seed=24,
                qk_norm=1, joint_rope=1),
    "K3n": _cfg(kind=3, dtype="f32", n_layers=2, hidden=256, n_heads=2, head_dim=128, mlp_dim=640,
                seq_img=204, grid_h=12, grid_w=17, n_patches=3, text_len=21, w_std="fan_in", seed=25, qk_norm=1),
    "C3n": _cfg(kind=2, dtype="bf16", n_layers=2, hidden=256, n_heads=4, head_dim=64, mlp_dim=1024,
                seq_img=1080, grid_h=30, grid_w=36, n_patches=4, text_len=77, seed=26, qk_norm=1, joint_rope=1),
    "C4n": _cfg(kind=3, dtype="bf16", n_layers=2, hidden=384, n_heads=3, head_dim=128, mlp_dim=1536,
                seq_img=1500, grid_h=30, grid_w=50, n_patches=5, text_len=45, seed=27, qk_norm=1),
    # final joint block of an MMDiT as the stage's last layer: its text stream only supplies keys and values
    "K2p": _cfg(kind=2, dtype="f32", n_layers=2, hidden=128, n_heads=2, head_dim=64, mlp_dim=320,
                seq_img=198, grid_h=11, grid_w=18, n_patches=3, text_len=29, w_std="fan_in", seed=30,
                txt_pre_only_last=1),
    "C3p": _cfg(kind=2, dtype="bf16", n_layers=2, hidden=256, n_heads=4, head_dim=64, mlp_dim=1024,
                seq_img=1080, grid_h=30, grid_w=36, n_patches=4, text_len=77, seed=31, qk_norm=1, txt_pre_only_last=1),
    # hidden size a multiple of 64: every GEMM of the block, the cross-attention projections included, takes the
    # direct-to-LDS kernels (C2s / C5s have K = 288 and fall back to the register-staged GEMM)
    "C2x": _cfg(kind=1, dtype="bf16", n_layers=2, hidden=576, n_heads=8, head_dim=72, mlp_dim=1152,
                seq_img=1200, grid_h=30, grid_w=40, n_patches=4, text_len=37, cross_dim=160, seed=29),
    "C3r": _cfg(kind=2, dtype="bf16", n_layers=2, hidden=256, n_heads=4, head_dim=64, mlp_dim=1024,
                seq_img=1080, grid_h=30, grid_w=36, n_patches=4, text_len=77, seed=28, joint_rope=1),
}


def patch_rows(cfg):
    """n: image tokens per patch."""
    return cfg["seq_img"] // cfg["n_patches"]


def joint_text_rows(cfg):
    """Text rows that live in the self-attention K/V buffer (joint-attention kinds only)."""
    return cfg["text_len"] if cfg["kind"] in (KIND_MMDIT_JOINT, KIND_SINGLE_STREAM) else 0


def kv_rows(cfg):
    """Lkv: rows of the per-layer K/V buffer."""
    return cfg["seq_img"] + joint_text_rows(cfg)


def round_to_bf16(a):
    """Round float32 values to the nearest bf16-representable value (ties to even).

    Storage-format conversion only; the result is still a float32 array.
    """
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = (u + bias) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def _store(cfg, a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return round_to_bf16(a) if cfg["dtype"] == "bf16" else a


def _normal(rng, shape, std=1.0):
    return (rng.standard_normal(shape, dtype=np.float32) * np.float32(std)).astype(np.float32)


def _linear(cfg, rng, out_f, in_f):
    """Weight [out, in] and bias [out]; std 0.02 or 1/sqrt(fan_in) as the config says."""
    std = (1.0 / np.sqrt(in_f)) if cfg["w_std"] == "fan_in" else float(cfg["w_std"])
    return _store(cfg, _normal(rng, (out_f, in_f), std)), _store(cfg, _normal(rng, (out_f,), std))


def _stream_weights(cfg, rng):
    """One weight stream of one layer.  All matrices are [out_features, in_features]."""
    d, F, kind = cfg["hidden"], cfg["mlp_dim"], cfg["kind"]
    w = {}
    if kind == KIND_ADALN_SINGLE_XATTN:
        std = (1.0 / np.sqrt(d)) if cfg["w_std"] == "fan_in" else float(cfg["w_std"])
        w["w_mod"] = _store(cfg, _normal(rng, (6, d), std))      # per-layer table added to cond
    elif kind == KIND_SINGLE_STREAM:
        w["w_mod"], w["b_mod"] = _linear(cfg, rng, 3 * d, d)
    else:
        w["w_mod"], w["b_mod"] = _linear(cfg, rng, 6 * d, d)
    w["w_qkv"], w["b_qkv"] = _linear(cfg, rng, 3 * d, d)
    g = float(cfg.get("qk_gain", 1.0))
    if g != 1.0:   # power-of-two gains keep bf16 values exact; peaks the softmax
        w["w_qkv"][: 2 * d] *= np.float32(g)
        w["b_qkv"][: 2 * d] *= np.float32(g)
    if kind != KIND_SINGLE_STREAM:
        w["w_o"], w["b_o"] = _linear(cfg, rng, d, d)
    w["w_up"], w["b_up"] = _linear(cfg, rng, F, d)
    if kind == KIND_SINGLE_STREAM:
        w["w_down"], w["b_down"] = _linear(cfg, rng, d, d + F)   # acts on [attn | GELU(mlp)]
    else:
        w["w_down"], w["b_down"] = _linear(cfg, rng, d, F)
    if kind == KIND_ADALN_SINGLE_XATTN:
        w["xattn_wq"], w["xattn_bq"] = _linear(cfg, rng, d, d)
        w["xattn_wkv"], w["xattn_bkv"] = _linear(cfg, rng, 2 * d, cfg["cross_dim"])
        w["xattn_wo"], w["xattn_bo"] = _linear(cfg, rng, d, d)
    if cfg.get("qk_norm"):   # learned per-channel scales of the q / k RMSNorm, shared by the heads (drawn last)
        w["q_norm_w"] = _store(cfg, 1.0 + 0.25 * _normal(rng, (cfg["head_dim"],)))
        w["k_norm_w"] = _store(cfg, 1.0 + 0.25 * _normal(rng, (cfg["head_dim"],)))
    return w


def make_weights(cfg, n_layers=None):
    """List (one entry per layer) of dicts of float32 arrays; kind 2 layers carry a 'txt' sub-dict."""
    rng = np.random.Generator(np.random.Philox(key=int(cfg["seed"]) * 1000 + 1))
    layers = []
    nl = cfg["n_layers"] if n_layers is None else n_layers
    for l in range(nl):
        w = _stream_weights(cfg, rng)
        if cfg["kind"] == KIND_MMDIT_JOINT:
            w["txt"] = _stream_weights(cfg, rng)
            if cfg.get("txt_pre_only_last") and l == nl - 1:
                # final joint block: the text stream keeps only what produces its keys and values (modulation with two
                # chunks [shift, scale], the QKV projection and the q / k norm scales)
                t = w["txt"]
                d = cfg["hidden"]
                w["txt"] = {k: v for k, v in t.items() if k in ("w_qkv", "b_qkv", "q_norm_w", "k_norm_w")}
                w["txt"]["w_mod"], w["txt"]["b_mod"] = t["w_mod"][: 2 * d].copy(), t["b_mod"][: 2 * d].copy()
        layers.append(w)
    return layers


def make_activations(cfg, noise=0.05):
    """x, x_prev [L,d]; cond; text; all float32 (bf16-representable when dtype is bf16).

    cond is [d] (kinds 0, 2, 3) or [6d] (kind 1).  text is [T, cross_dim] for
    kind 1 (keys of the cross-attention) and [T, d] for kinds 2, 3 (joint rows).
    """
    rng = np.random.Generator(np.random.Philox(key=int(cfg["seed"]) * 1000 + 2))
    L, d, T, kind = cfg["seq_img"], cfg["hidden"], cfg["text_len"], cfg["kind"]
    out = {}
    out["x"] = _store(cfg, _normal(rng, (L, d)))
    out["x_prev"] = _store(cfg, out["x"] + np.float32(noise) * _normal(rng, (L, d)))
    if kind == KIND_ADALN_SINGLE_XATTN:
        # adaLN-single: the stage receives the model-global 6d projection of the conditioning embedding, not
        # the embedding itself.  It is drawn at the scale that projection has under the workload's own weight
        # distribution, std(W) * sqrt(d) * rms(SiLU(c)) with rms(SiLU(c)) ~ 0.55 std(c): the same scale the
        # other kinds' per-layer modulation Linear produces from their embedding.
        w_std = (1.0 / np.sqrt(d)) if cfg["w_std"] == "fan_in" else float(cfg["w_std"])
        out["cond"] = _store(cfg, _normal(rng, (6 * d,), w_std * np.sqrt(d) * 0.55 * cfg["cond_std"]))
    else:
        out["cond"] = _store(cfg, _normal(rng, (d,), cfg["cond_std"]))
    if kind == KIND_ADALN_SINGLE_XATTN:
        out["text"] = _store(cfg, _normal(rng, (T, cfg["cross_dim"])))
    elif kind in (KIND_MMDIT_JOINT, KIND_SINGLE_STREAM):
        out["text"] = _store(cfg, _normal(rng, (T, d)))
    else:
        out["text"] = None
    return out


def make_kv_fill(cfg, layer, std=1.0):
    """Synthetic stale K and V rows [Lkv, d] for one layer, for tests that fill the
    caller-owned buffer directly instead of running the warm-up pass."""
    rng = np.random.Generator(np.random.Philox(key=int(cfg["seed"]) * 1000 + 100 + layer))
    Lkv, d = kv_rows(cfg), cfg["hidden"]
    return _store(cfg, _normal(rng, (Lkv, d), std)), _store(cfg, _normal(rng, (Lkv, d), std))


def variant(cfg, **kw):
    c = dict(cfg)
    c.update(kw)
    return _cfg(**c)


def make_sampling(cfg, steps, dt_total=-0.2, cond_drift=0.1):
    """Inputs of an S-step sampling loop: per-step conditioning vectors (the timestep embedding drifts from step to
    step; a fixed part plus a per-step part of relative size cond_drift) and per-step Euler step sizes that sum to
    dt_total.  Float32, bf16-representable for bf16 workloads."""
    rng = np.random.Generator(np.random.Philox(key=int(cfg["seed"]) * 1000 + 3))
    base = make_activations(cfg)["cond"]
    scale = float(np.sqrt(np.mean(base.astype(np.float64) ** 2)))
    conds = [_store(cfg, base + np.float32(cond_drift * scale) * _normal(rng, base.shape)) for _ in range(steps)]
    w = 1.0 + 0.5 * np.cos(np.arange(steps))          # uneven steps, as real noise schedules have
    dts = [float(dt_total * wi / w.sum()) for wi in w]
    return conds, dts


def split_stages(layers, n_stages):
    """Consecutive, equal-sized groups of layers (one group per pipeline stage)."""
    per = len(layers) // n_stages
    assert per * n_stages == len(layers)
    return [layers[i * per:(i + 1) * per] for i in range(n_stages)]
