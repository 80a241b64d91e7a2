"""Pins for the CPU oracle: what the method and the mathematics fix, checked against
something other than the oracle itself (library routines, scalar brute force, closed forms).

The paper prints no numeric value for the patch-stage path, so the pins are the invariants of
PipeFusion, Sec. 3.3: one patch (M = 1) or a buffer that is fresh everywhere must reproduce the
original model exactly; App. B: a zero-initialised buffer has a closed form.
"""
import math

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import pf_oracle as po
from full_forward_ref import full_forward

FP32_TWINS = ["K0f", "K1f", "K2f", "K3f", "K2n", "K3n", "K2p"]   # K2n / K3n: q,k RMSNorm (and RoPE on the two-stream block); K2p: final joint block
RTOL = 1e-9


def _rel(a, b):
    return float(np.max(np.abs(a - b)) / (np.sqrt(np.mean(b ** 2)) + 1e-300))


def _setup(name, **kw):
    cfg = wl.variant(wl.CONFIGS[name], **kw) if kw else wl.CONFIGS[name]
    return cfg, wl.make_weights(cfg), wl.make_activations(cfg)


# ---- I1: M = 1 is the original model -------------------------------------------------------
@pytest.mark.parametrize("name", FP32_TWINS)
def test_single_patch_equals_full_forward(name):
    cfg, W, A = _setup(name, n_patches=1)
    o = po.StageOracle(cfg, W)
    o.kv_init(None, text=A["text"] if cfg["kind"] == 1 else None)
    # poison the buffers: with M = 1 every row is rewritten before it is attended to
    for l in range(o.nl):
        o.kbuf[l][:] = 7.0
        o.vbuf[l][:] = -3.0
    txt = A["text"] if cfg["kind"] in (2, 3) else None
    got = o.patch_forward(A["x"], A["cond"], 0, text=txt)
    ref_y, ref_t = full_forward(cfg, W, A["x"], A["cond"], A["text"])
    if txt is not None:
        assert _rel(got[1], ref_t) < RTOL
        got = got[0]
    assert _rel(got, ref_y) < RTOL


# ---- I2: fresh-everywhere buffer -------------------------------------------------------------
@pytest.mark.parametrize("name", FP32_TWINS)
def test_fresh_buffer_equals_full_forward_rows(name):
    cfg, W, A = _setup(name)
    o = po.StageOracle(cfg, W)
    warm = o.kv_init(A["x"], A["cond"], text=A["text"])
    ref_y, ref_t = full_forward(cfg, W, A["x"], A["cond"], A["text"])
    assert _rel(warm[0], ref_y) < RTOL                  # the warm-up pass itself is the exact model
    if ref_t is not None:
        assert _rel(warm[1], ref_t) < RTOL
    n = wl.patch_rows(cfg)
    for p in reversed(range(cfg["n_patches"])):        # any order
        y = o.patch_forward(A["x"][p * n:(p + 1) * n], A["cond"], p)   # image rows only
        assert _rel(y, ref_y[p * n:(p + 1) * n]) < RTOL
    if cfg["kind"] in (2, 3):                           # text rows ride along with patch 0
        y, yt = o.patch_forward(A["x"][:n], A["cond"], 0, text=A["text"])
        assert _rel(y, ref_y[:n]) < RTOL and _rel(yt, ref_t) < RTOL


def test_stale_buffer_differs_and_error_shrinks_with_noise():
    """Sanity (not a gate): with x != x_prev the output is an approximation whose error scales with
    the step-to-step difference (input temporal redundancy, Sec. 2)."""
    cfg, W, _ = _setup("K0f")
    errs = []
    for noise in (0.2, 0.05, 0.0):
        A = wl.make_activations(cfg, noise=noise)
        o = po.StageOracle(cfg, W)
        o.kv_init(A["x_prev"], A["cond"])
        ref_y, _ = full_forward(cfg, W, A["x"], A["cond"])
        n = wl.patch_rows(cfg)
        errs.append(_rel(o.patch_forward(A["x"][:n], A["cond"], 0), ref_y[:n]))
    assert errs[0] > errs[1] > errs[2] and errs[2] < RTOL


# ---- I4: scalar brute force on a tiny stage ---------------------------------------------------
def _bf_linear(x, w, b):
    return [sum(xi * wij for xi, wij in zip(x, wrow)) + bi for wrow, bi in zip(w, b)]


def _bf_ln_mod(x, shift, scale, eps):
    d = len(x)
    mu = sum(x) / d
    var = sum((v - mu) ** 2 for v in x) / d
    return [(v - mu) / math.sqrt(var + eps) * (1 + sc) + sh for v, sh, sc in zip(x, shift, scale)]


def _bf_gelu(v):
    return 0.5 * v * (1 + math.tanh(math.sqrt(2 / math.pi) * (v + 0.044715 * v ** 3)))


def _bf_block(xrows, row0, K, V, w, mod, H, eps):
    """One adaLN-zero block on the given rows; K, V are lists of rows (mutated: write before attend)."""
    d = len(xrows[0])
    dh = d // H
    qs = []
    for i, x in enumerate(xrows):
        qkv = _bf_linear(_bf_ln_mod(x, mod[0], mod[1], eps), w["w_qkv"], w["b_qkv"])
        qs.append(qkv[:d])
        K[row0 + i] = qkv[d:2 * d]
        V[row0 + i] = qkv[2 * d:]
    out = []
    for x, q in zip(xrows, qs):
        a = [0.0] * d
        for h in range(H):
            s = [sum(q[h * dh + c] * Kj[h * dh + c] for c in range(dh)) / math.sqrt(dh) for Kj in K]
            mx = max(s)
            e = [math.exp(v - mx) for v in s]
            z = sum(e)
            for c in range(dh):
                a[h * dh + c] = sum(ej * Vj[h * dh + c] for ej, Vj in zip(e, V)) / z
        o = _bf_linear(a, w["w_o"], w["b_o"])
        x = [xv + g * ov for xv, g, ov in zip(x, mod[2], o)]
        u = [_bf_gelu(v) for v in _bf_linear(_bf_ln_mod(x, mod[3], mod[4], eps), w["w_up"], w["b_up"])]
        dn = _bf_linear(u, w["w_down"], w["b_down"])
        out.append([xv + g * dv for xv, g, dv in zip(x, mod[5], dn)])
    return out


def test_brute_force_tiny_stage():
    cfg = wl.variant(wl.CONFIGS["K0f"], hidden=8, n_heads=2, head_dim=4, mlp_dim=12, seq_img=6,
                     grid_h=2, grid_w=3, n_patches=3, n_layers=2, seed=5)
    W, A = wl.make_weights(cfg), wl.make_activations(cfg, noise=0.3)
    Wl = [{k: v.astype(np.float64).tolist() for k, v in w.items()} for w in W]
    d, H, L, n, eps = 8, 2, 6, 2, cfg["ln_eps"]
    cond = A["cond"].astype(np.float64).tolist()
    sc = [c / (1 + math.exp(-c)) for c in cond]
    mods = []
    for w in Wl:
        m = _bf_linear(sc, w["w_mod"], w["b_mod"])
        mods.append([m[i * d:(i + 1) * d] for i in range(6)])
    # warm-up: whole previous-step sequence, exact
    K = [[None] * L for _ in Wl]
    V = [[None] * L for _ in Wl]
    rows = A["x_prev"].astype(np.float64).tolist()
    for l, w in enumerate(Wl):
        rows = _bf_block(rows, 0, K[l], V[l], w, mods[l], H, eps)
    o = po.StageOracle(cfg, W)
    warm, _ = o.kv_init(A["x_prev"], A["cond"])
    assert _rel(warm, np.array(rows)) < 1e-10
    # then patches 1, 0, 2 of the new step, stale rows elsewhere
    for p in (1, 0, 2):
        rows = A["x"][p * n:(p + 1) * n].astype(np.float64).tolist()
        for l, w in enumerate(Wl):
            rows = _bf_block(rows, p * n, K[l], V[l], w, mods[l], H, eps)
        y = o.patch_forward(A["x"][p * n:(p + 1) * n], A["cond"], p)
        assert _rel(y, np.array(rows)) < 1e-10
        for l in range(2):
            assert _rel(o.kbuf[l], np.array(K[l])) < 1e-10
            assert _rel(o.vbuf[l], np.array(V[l])) < 1e-10


# ---- I5: zero-initialised buffer closed form --------------------------------------------------
def test_zero_buffer_closed_form():
    rng = np.random.default_rng(3)
    H, dh, n, Lkv, off = 2, 8, 5, 23, 10
    d = H * dh
    q, k, v = (rng.standard_normal((n, d)) for _ in range(3))
    K = np.zeros((Lkv, d))
    V = np.zeros((Lkv, d))
    K[off:off + n], V[off:off + n] = k, v
    got = po.attention(q, K, V, H)
    for h in range(H):
        sl = slice(h * dh, (h + 1) * dh)
        e = np.exp(q[:, sl] @ k[:, sl].T / math.sqrt(dh))            # stale rows: score 0 -> e^0 = 1
        want = (e @ v[:, sl]) / (e.sum(1, keepdims=True) + (Lkv - n))
        assert np.allclose(got[:, sl], want, rtol=1e-12, atol=1e-14)


def test_zero_init_stage_buffers_are_zero_outside_patch():
    cfg, W, A = _setup("K1f")
    o = po.StageOracle(cfg, W)
    o.kv_init(None, text=A["text"])
    n = wl.patch_rows(cfg)
    o.patch_forward(A["x"][n:2 * n], A["cond"], 1)
    for l in range(o.nl):
        for buf in (o.kbuf[l], o.vbuf[l]):
            assert not buf[:n].any() and not buf[2 * n:].any() and buf[n:2 * n].any()


# ---- I3: softmax ---------------------------------------------------------------------------
def test_softmax_rows_sum_to_one_even_when_peaked():
    rng = np.random.default_rng(0)
    q = rng.standard_normal((7, 16)) * 30
    k = rng.standard_normal((11, 16)) * 30
    v = rng.standard_normal((11, 16))
    out, probs = po.attention(q, k, v, 2, return_probs=True)
    for p in probs:
        assert (p >= 0).all() and np.allclose(p.sum(1), 1.0, atol=1e-12)
    # a convex combination stays inside the values' range, head by head
    for h in range(2):
        sl = slice(h * 8, (h + 1) * 8)
        assert (out[:, sl] <= v[:, sl].max(0) + 1e-12).all() and (out[:, sl] >= v[:, sl].min(0) - 1e-12).all()


def test_attention_matches_library_sdpa():
    rng = np.random.default_rng(1)
    H, dh = 3, 72
    q, k, v = rng.standard_normal((9, H * dh)), rng.standard_normal((31, H * dh)), rng.standard_normal((31, H * dh))
    tq, tk, tv = (torch.tensor(t).view(t.shape[0], H, dh).transpose(0, 1) for t in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv).transpose(0, 1).reshape(9, H * dh).numpy()
    assert np.allclose(po.attention(q, k, v, H), ref, rtol=1e-11, atol=1e-13)


# ---- I8: LayerNorm / GELU / SiLU / RoPE identities ---------------------------------------------
def test_layernorm_identities_and_library():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((5, 48)) * 3 + 1.5
    y = po.layer_norm(x, 1e-6)
    assert np.allclose(y.mean(1), 0, atol=1e-12)
    assert np.allclose(y.var(1), x.var(1) / (x.var(1) + 1e-6), rtol=1e-12)
    ref = torch.nn.functional.layer_norm(torch.tensor(x), (48,), eps=1e-6).numpy()
    assert np.allclose(y, ref, rtol=1e-12, atol=1e-13)
    sh, sc = rng.standard_normal(48), rng.standard_normal(48)
    assert np.allclose(po.ln_modulate(x, sh, sc, 1e-6), ref * (1 + sc) + sh, rtol=1e-12, atol=1e-12)
    # shift/scale are not swapped: scale = -1 kills the normalised term
    assert np.allclose(po.ln_modulate(x, sh, -np.ones(48), 1e-6), np.broadcast_to(sh, x.shape), atol=1e-12)


def test_gelu_silu_identities_and_library():
    x = np.linspace(-6, 6, 241)
    for tanh in (True, False):
        g = po.gelu(x, tanh)
        assert g[120] == 0.0
        assert np.allclose(g - po.gelu(-x, tanh), x, atol=1e-12)          # GELU(x) - GELU(-x) = x
        assert abs(po.gelu(np.array([30.0]), tanh)[0] - 30.0) < 1e-12
        ref = torch.nn.functional.gelu(torch.tensor(x), approximate="tanh" if tanh else "none").numpy()
        assert np.allclose(g, ref, rtol=1e-12, atol=1e-14)
    assert np.max(np.abs(po.gelu(x, True) - po.gelu(x, False))) > 1e-4      # the two flavours do differ
    assert np.allclose(po.silu(x), torch.nn.functional.silu(torch.tensor(x)).numpy(), rtol=1e-12, atol=1e-14)


def test_rope_norm_relative_position_and_complex_form():
    rng = np.random.default_rng(4)
    H, dh, theta = 2, 16, 1e4
    q, k = rng.standard_normal((1, H * dh)), rng.standard_normal((1, H * dh))

    def rot(t, r, c):
        return po.rope_apply(t, po.rope_angles([r], [c], dh, theta), H)

    assert np.allclose(np.linalg.norm(rot(q, 5, 9)), np.linalg.norm(q), rtol=1e-13)
    assert np.allclose(rot(q, 0, 0), q, atol=0)                               # position (0,0): identity
    base = [float(rot(q, 3, 4)[0, h * dh:(h + 1) * dh] @ rot(k, 1, 7)[0, h * dh:(h + 1) * dh]) for h in range(H)]
    for dr, dc in ((2, 0), (0, 11), (6, 5)):
        sh = [float(rot(q, 3 + dr, 4 + dc)[0, h * dh:(h + 1) * dh] @ rot(k, 1 + dr, 7 + dc)[0, h * dh:(h + 1) * dh])
              for h in range(H)]
        assert np.allclose(sh, base, rtol=1e-10, atol=1e-12)
    # row position must only touch the first half of the head's channels, column the second half
    assert np.allclose(rot(q, 9, 0)[0, dh // 2:dh], q[0, dh // 2:dh]) and not np.allclose(rot(q, 9, 0)[0, :dh // 2], q[0, :dh // 2])
    assert np.allclose(rot(q, 0, 9)[0, :dh // 2], q[0, :dh // 2])
    # first pair of an axis turns by exactly pos radians (frequency theta^0 = 1)
    v = np.zeros((1, H * dh)); v[0, 0] = 1.0
    r = rot(v, 2, 0)
    assert np.allclose(r[0, :2], [math.cos(2.0), math.sin(2.0)], atol=1e-14)
    # last pair of an axis: theta^(-(w-2)/w) with w = dh/2
    v = np.zeros((1, H * dh)); v[0, dh // 2 - 2] = 1.0
    w = dh // 2
    ang = 3.0 * theta ** (-(w - 2) / w)
    assert np.allclose(rot(v, 3, 0)[0, dh // 2 - 2:dh // 2], [math.cos(ang), math.sin(ang)], atol=1e-14)


# ---- I9 / I10 / I6 / I7 -------------------------------------------------------------------------
def test_qk_rmsnorm_identities_and_library():
    """RMSNorm per head: unit weights give unit rms per (row, head); the output does not depend on the scale of the
    input; torch's rms_norm agrees; a head-wise permutation of rows commutes with it."""
    rng = np.random.default_rng(3)
    n, H, dh = 7, 3, 64
    t = rng.normal(size=(n, H * dh)) * rng.uniform(0.1, 9.0, size=(n, 1))
    w = 1.0 + 0.3 * rng.normal(size=dh)
    unit = po.rms_norm_heads(t, np.ones(dh), H, 0.0).reshape(n, H, dh)
    assert np.allclose(np.sqrt(np.mean(unit ** 2, axis=-1)), 1.0, atol=1e-12)
    a, b = po.rms_norm_heads(t, w, H, 0.0), po.rms_norm_heads(37.5 * t, w, H, 0.0)
    assert np.allclose(a, b, rtol=1e-12, atol=1e-12)
    ref = torch.nn.functional.rms_norm(torch.as_tensor(t).view(n, H, dh), (dh,), weight=torch.as_tensor(w), eps=1e-6)
    assert np.allclose(po.rms_norm_heads(t, w, H, 1e-6), ref.reshape(n, H * dh).numpy(), rtol=1e-12, atol=1e-12)
    # a zero row stays finite with eps > 0
    z = po.rms_norm_heads(np.zeros((2, H * dh)), w, H, 1e-6)
    assert np.all(z == 0.0)


def test_qk_norm_changes_the_result_and_bounds_the_scores():
    """The flag is live: switching it off changes the output; with it on, every attention score is bounded by
    dh * max|wq| * max|wk| / sqrt(dh) (Cauchy-Schwarz on unit-rms vectors), whatever the gain of the projection."""
    cfg = wl.variant(wl.CONFIGS["K3n"], qk_gain=16.0)
    W, A = wl.make_weights(cfg), wl.make_activations(cfg)
    o = po.StageOracle(cfg, W)
    warm, _ = o.kv_init(A["x"], A["cond"], text=A["text"])
    off = po.StageOracle(dict(cfg, qk_norm=0), W)
    warm_off, _ = off.kv_init(A["x"], A["cond"], text=A["text"])
    assert _rel(warm, warm_off) > 1e-3
    H, dh = cfg["n_heads"], cfg["head_dim"]
    K = o.kbuf[0].reshape(-1, H, dh)
    bound = np.sqrt(dh) * np.max(np.abs(W[0]["k_norm_w"]))
    assert np.all(np.sqrt(np.sum(K * K, axis=-1)) <= bound * (1 + 1e-9))     # |k_h| <= sqrt(dh) * max|w| (RoPE keeps norms)


def test_zero_gates_make_the_stage_identity_but_still_write_kv():
    cfg, W, A = _setup("K0f")
    d = cfg["hidden"]
    for w in W:
        for blk in (2, 5):
            w["w_mod"][blk * d:(blk + 1) * d] = 0
            w["b_mod"][blk * d:(blk + 1) * d] = 0
    o = po.StageOracle(cfg, W)
    o.kv_init(None)
    n = wl.patch_rows(cfg)
    y = o.patch_forward(A["x"][:n], A["cond"], 0)
    assert np.array_equal(y, A["x"][:n].astype(np.float64))
    assert o.kbuf[1][:n].any() and o.vbuf[1][:n].any()


def test_permuting_stale_rows_leaves_attention_unchanged():
    rng = np.random.default_rng(6)
    q, k, v = rng.standard_normal((4, 24)), rng.standard_normal((50, 24)), rng.standard_normal((50, 24))
    perm = rng.permutation(50)
    assert np.allclose(po.attention(q, k, v, 3), po.attention(q, k[perm], v[perm], 3), rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("name", ["K0f", "K2f", "K3f"])
def test_untouched_rows_and_sweep_refresh(name):
    cfg, W, A = _setup(name)
    o = po.StageOracle(cfg, W)
    o.kv_init(A["x_prev"], A["cond"], text=A["text"])
    n, Tj = wl.patch_rows(cfg), wl.joint_text_rows(cfg)
    before = [(o.kbuf[l].copy(), o.vbuf[l].copy()) for l in range(o.nl)]
    p = 1
    o.patch_forward(A["x"][p * n:(p + 1) * n], A["cond"], p)
    lo, hi = Tj + p * n, Tj + (p + 1) * n
    for l in range(o.nl):
        for new, old in zip((o.kbuf[l], o.vbuf[l]), before[l]):
            assert np.array_equal(new[:lo], old[:lo]) and np.array_equal(new[hi:], old[hi:])
            assert not np.array_equal(new[lo:hi], old[lo:hi])
    # full sweep: afterwards every image row block is the fresh one of its own call
    o.kv_init(A["x_prev"], A["cond"], text=A["text"])
    stale = [o.kbuf[l].copy() for l in range(o.nl)]
    for p in range(cfg["n_patches"]):
        o.patch_forward(A["x"][p * n:(p + 1) * n], A["cond"], p)
    for l in range(o.nl):
        assert not np.any(np.all(o.kbuf[l][Tj:] == stale[l][Tj:], axis=1))     # all image rows rewritten
        assert np.array_equal(o.kbuf[l][:Tj], stale[l][:Tj])                   # text rows untouched without text


def test_kv_memory_footprint_formula():
    """Sec. 3.4, Table 1: a stage holds full-sequence K and V for its own layers only."""
    for name in ("C2", "C3", "C4", "C5"):
        cfg = wl.CONFIGS[name]
        o_rows = wl.kv_rows(cfg)
        assert o_rows == cfg["seq_img"] + (cfg["text_len"] if cfg["kind"] in (2, 3) else 0)


def test_bf16_storage_rounding_matches_torch():
    a = (np.random.default_rng(0).standard_normal(10000) * 3).astype(np.float32)
    ref = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(wl.round_to_bf16(a), ref)
