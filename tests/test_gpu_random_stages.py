"""Seeded random stage configurations against the CPU oracle (GPU).

The named twins cover each block kind and flag once; here kind, head size, head count, layer count, sequence and
patch sizes, text length, batch and the optional flags (q/k norm, RoPE on the two-stream block, final joint block)
are drawn together, so that combinations nobody wrote down get a parity run: a warm-up pass, then every patch of
the next step in a drawn order, outputs compared image by image."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle.pf_oracle import StageOracle

pytestmark = pytest.mark.gpu
TOL = {"f32": 1e-4, "bf16": 2e-2}


def _f32(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def _relerr(got, ref):
    got = got.detach().double().cpu().numpy()
    return float(np.max(np.abs(got - ref)) / (np.sqrt(np.mean(ref ** 2)) + 1e-30))


def _draw_config(i):
    rng = np.random.Generator(np.random.Philox(key=909000 + i))
    kind = int(rng.integers(0, 4))
    dtype = "bf16" if rng.random() < 0.6 else "f32"
    dh = int(rng.choice([64, 72, 128, 40])) if kind != 3 else int(rng.choice([64, 128, 72, 40]))
    qk_norm = int(kind in (2, 3) and rng.random() < 0.5)
    if qk_norm:
        dh = int(rng.choice([64, 128, 32]))                      # the per-head RMSNorm wants a power of two
    H = int(rng.integers(1, 5))
    d = H * dh
    gh, gw = int(rng.integers(3, 30)), int(rng.integers(3, 30))
    L = gh * gw
    divs = [m for m in range(1, 9) if L % m == 0]
    M = int(rng.choice(divs))
    cfg = dict(kind=kind, dtype=dtype, n_layers=int(rng.integers(1, 4)), hidden=d, n_heads=H, head_dim=dh,
               mlp_dim=int(rng.integers(2, 12)) * 32, seq_img=L, grid_h=gh, grid_w=gw, n_patches=M,
               seed=4000 + i, qk_norm=qk_norm)
    cfg["w_std"] = "fan_in" if dtype == "f32" else 0.02
    cfg["cond_std"] = None                                       # the workload module's default for the dtype
    if kind in (1, 2, 3):
        cfg["text_len"] = int(rng.integers(1, 90))
    if kind == 1:
        cfg["cross_dim"] = int(rng.integers(2, 20)) * 8
    if kind == 2:
        cfg["joint_rope"] = int(rng.random() < 0.4 and dh % 4 == 0)
        cfg["txt_pre_only_last"] = int(rng.random() < 0.4)
    B = int(rng.choice([1, 1, 2, 3]))
    return wl.variant(wl.CONFIGS["C1"], **cfg), B, rng


@pytest.mark.parametrize("i", list(range(48)))
def test_random_stage_configuration(i):
    from paper_2405_14430_amd import Stage
    cfg, B, rng = _draw_config(i)
    kind, joint = cfg["kind"], cfg["kind"] in (2, 3)
    tol = TOL[cfg["dtype"]]
    print("random stage", i, {k: cfg[k] for k in ("kind", "dtype", "n_layers", "hidden", "n_heads", "head_dim", "mlp_dim",
                                                  "seq_img", "n_patches", "text_len", "qk_norm", "joint_rope",
                                                  "txt_pre_only_last")}, "B", B, flush=True)
    W = wl.make_weights(cfg)
    acts = [wl.make_activations(wl.variant(cfg, seed=cfg["seed"] + 100 * b)) for b in range(B)]
    stack = lambda key: np.stack([a[key] for a in acts], axis=0) if B > 1 else acts[0][key]
    st = Stage(dict(cfg, batch=B), W)
    orcs = [StageOracle(cfg, W) for _ in range(B)]
    cond = _f32(stack("cond"))
    text = None
    if kind == 1:
        text = _f32(stack("text")).to(st.dt)
    elif joint:
        text = _f32(stack("text"))
    pick = (lambda t, b: t[b]) if B > 1 else (lambda t, b: t)

    y0, t0 = st.kv_init(_f32(stack("x_prev")), cond, text, want_output=True)
    torch.cuda.synchronize()
    for b in range(B):
        ref0, reft0 = orcs[b].kv_init(acts[b]["x_prev"], acts[b]["cond"], text=acts[b]["text"])
        assert _relerr(pick(y0, b), ref0) < tol, ("warm-up", b)
        if joint:
            assert _relerr(pick(t0, b), reft0) < tol, ("warm-up text", b)

    n = wl.patch_rows(cfg)
    order = list(rng.permutation(cfg["n_patches"]))
    with_text = joint and rng.random() < 0.7
    for j, p in enumerate(order):
        xp = _f32(np.stack([a["x"][p * n:(p + 1) * n] for a in acts], axis=0) if B > 1 else acts[0]["x"][p * n:(p + 1) * n])
        carry = with_text and j == 0                      # the text rows ride with the first call of the step
        same = j > 0 and rng.random() < 0.5               # the step's later calls may keep the modulation vectors
        if carry:
            y, yt = st.patch_forward(xp, cond, int(p), text=text)
        else:
            y, yt = st.patch_forward(xp, cond, int(p), same_cond=same), None
        torch.cuda.synchronize()
        for b in range(B):
            a = acts[b]
            if carry:
                ref, reft = orcs[b].patch_forward(a["x"][p * n:(p + 1) * n], a["cond"], int(p), text=a["text"])
                assert _relerr(pick(yt, b), reft) < tol, ("text", int(p), b)
            else:
                ref = orcs[b].patch_forward(a["x"][p * n:(p + 1) * n], a["cond"], int(p))
            assert _relerr(pick(y, b), ref) < tol, ("patch", int(p), b)
    st.destroy()
