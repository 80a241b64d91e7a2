"""Parity at the full sizes of the named workloads (GPU), in the launch configuration bench.py times.

C2 and C3 run their real warm-up pass on both sides.  For C4 and C5 the oracle's warm-up pass alone would be tens of
Tflop of float64 work, so the caller-owned K/V buffer is filled directly with seeded synthetic stale rows on both sides
(the buffer contents are inputs to a patch call, wherever they came from) and single calls are compared at the
configured depth: about a minute of float64 oracle work each.
"""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle.pf_oracle import StageOracle

pytestmark = pytest.mark.gpu
TOL = 2e-2


def _pkg():
    import paper_2405_14430_amd as pkg
    return pkg


def _log(*a):
    print(*a, flush=True)


def _f32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def _relerr(got, ref):
    got = got.detach().double().cpu().numpy()
    return float(np.max(np.abs(got - ref)) / (np.sqrt(np.mean(ref ** 2)) + 1e-30))


def _rmserr(got, ref):
    got = got.detach().double().cpu().numpy()
    return float(np.sqrt(np.mean((got - ref) ** 2)) / (np.sqrt(np.mean(ref ** 2)) + 1e-30))


@pytest.mark.parametrize("name", ["C2", "C3"])
def test_full_size_with_real_warmup(name):
    cfg = wl.CONFIGS[name]
    W, A = wl.make_weights(cfg), wl.make_activations(cfg)
    st = _pkg().Stage(cfg, W)
    orc = StageOracle(cfg, W)
    cond = _f32(A["cond"])
    text = _f32(A["text"]).to(torch.bfloat16) if cfg["kind"] == 1 else _f32(A["text"])
    _log(name, "warm-up pass")
    y0, _ = st.kv_init(_f32(A["x_prev"]), cond, text, want_output=True)
    torch.cuda.synchronize()
    ref0, _ = orc.kv_init(A["x_prev"], A["cond"], text=A["text"])
    e0 = _relerr(y0, ref0)
    _log(f"  warm-up err {e0:.3e}")
    assert e0 < TOL
    n, M = wl.patch_rows(cfg), cfg["n_patches"]
    for p in (0, M - 1):
        xp = A["x"][p * n:(p + 1) * n]
        if cfg["kind"] == 2 and p == 0:
            y, yt = st.patch_forward(_f32(xp), cond, p, text=text)
            torch.cuda.synchronize()
            ref, reft = orc.patch_forward(xp, A["cond"], p, text=A["text"])
            assert _relerr(yt, reft) < TOL
        else:
            y = st.patch_forward(_f32(xp), cond, p)
            torch.cuda.synchronize()
            ref = orc.patch_forward(xp, A["cond"], p)
        err = _relerr(y, ref)
        _log(f"  {name} patch {p}: err {err:.3e}")
        assert err < TOL
    st.destroy()


# ---- C4 and C5 at their configured depth (7 and 4 layers), one oracle call per test -------------------------------
_BIG = {}
_LAST = {}      # rms error of the last call compared (the floor test reads it)


def _big(name, cond_std=None):
    """Stage, oracle and inputs of a big workload, built once per (workload, conditioning std) and kept for the tests
    that use them; the previous one is dropped first (the float64 oracle of the 7-layer Flux-scale stage is ~14 GB)."""
    key = (name, cond_std)
    if key not in _BIG:
        for k in list(_BIG):
            _BIG.pop(k)[0].destroy()
        cfg = wl.CONFIGS[name] if cond_std is None else wl.variant(wl.CONFIGS[name], cond_std=cond_std)
        _log(name, "cond std", cfg["cond_std"], ": weights, stage, oracle")
        W, A = wl.make_weights(cfg), wl.make_activations(cfg)
        st = _pkg().Stage(cfg, W)
        orc = StageOracle(cfg, W)
        orc.on_layer = lambda l: _log("    oracle: layer", l, "done")
        if cfg["kind"] == 1:
            st.kv_init(None, None, _f32(A["text"]).to(torch.bfloat16))
            orc.kv_init(None, text=A["text"])
        else:
            st.kv_init(None)
            orc.kv_init(None)
        fills = [wl.make_kv_fill(cfg, l) for l in range(cfg["n_layers"])]
        _BIG[key] = (st, orc, cfg, A, fills)
    return _BIG[key]


def _refill(st, orc, cfg, fills):
    """Both sides get the same synthetic stale rows in every layer's buffer (what an earlier test wrote is gone)."""
    H, dh = cfg["n_heads"], cfg["head_dim"]
    for l, (k, v) in enumerate(fills):
        orc.set_kv(l, k, v)
        K, V, _ = st.kv_view(l)
        K.copy_(_f32(k).to(torch.bfloat16).view(-1, H, dh))
        V.copy_(_f32(v).to(torch.bfloat16).view(-1, H, dh))


def _one_call(name, p, with_text, cond_std=None):
    """One patch call at full size and full depth on both sides; returns the errors of y, the text rows and the fresh
    K rows, after checking bit for bit that no stale row of any layer's buffer changed."""
    st, orc, cfg, A, fills = _big(name, cond_std)
    _refill(st, orc, cfg, fills)
    n, Tj = wl.patch_rows(cfg), wl.joint_text_rows(cfg)
    xp = A["x"][p * n:(p + 1) * n]
    cond = _f32(A["cond"])
    _log(name, "patch", p, "with text rows" if with_text else "image only", "layers", cfg["n_layers"])
    et = None
    if with_text:
        y, yt = st.patch_forward(_f32(xp), cond, p, text=_f32(A["text"]))
        torch.cuda.synchronize()
        ref, reft = orc.patch_forward(xp, A["cond"], p, text=A["text"])
        et = _relerr(yt, reft)
    else:
        y = st.patch_forward(_f32(xp), cond, p)
        torch.cuda.synchronize()
        ref = orc.patch_forward(xp, A["cond"], p)
    err = _relerr(y, ref)
    _LAST["rms"] = _rmserr(y, ref)
    _log(f"  rms(err)/rms(y) = {_LAST['rms']:.3e}")
    lo, hi = Tj + p * n, Tj + (p + 1) * n
    keep = np.ones(wl.kv_rows(cfg), dtype=bool)
    keep[lo:hi] = False
    if with_text:
        keep[:Tj] = False
    idx = torch.from_numpy(np.nonzero(keep)[0]).cuda()
    ek = 0.0
    for l, (k, v) in enumerate(fills):
        K, V, _ = st.kv_view(l)
        assert torch.equal(K[idx].reshape(len(idx), -1), _f32(k).to(torch.bfloat16)[idx]), ("stale K rows changed", l)
        assert torch.equal(V[idx].reshape(len(idx), -1), _f32(v).to(torch.bfloat16)[idx]), ("stale V rows changed", l)
        for got, want in ((K[lo:hi], orc.kbuf[l][lo:hi]), (V[lo:hi], orc.vbuf[l][lo:hi])):
            g = got.double().cpu().numpy().reshape(n, -1)
            # stored in bf16: one storage rounding of the value plus the bar for the arithmetic in front of it
            excess = np.abs(g - want) - 2.0 ** -8 * np.abs(want)
            ek = max(ek, float(np.max(excess) / np.sqrt(np.mean(want ** 2))))
    _log(f"  {name} cond std {cfg['cond_std']} patch {p}: y err {err:.3e}" + (f", text rows {et:.3e}" if et is not None else "") +
         f", fresh K/V rows beyond storage rounding {ek:.3e}")
    return err, et, ek


@pytest.mark.timeout(900)
@pytest.mark.parametrize("name,p,with_text", [("C4", 0, True), ("C4", 7, False), ("C5", 0, False), ("C5", 15, False)])
def test_full_size_full_depth_on_synthetic_stale_buffer(name, p, with_text):
    """The configured depth (C4: 7 layers, C5: 4) at the configured size: the call with the joint text rows and the
    image-only call that the benchmark times (C4), first and last patch (C5)."""
    err, et, ek = _one_call(name, p, with_text)
    assert err < TOL and ek < TOL and (et is None or et < TOL)


@pytest.mark.timeout(900)
@pytest.mark.parametrize("name,cond_std", [("C4", 0.5), ("C4", 1.0), ("C3", 1.0), ("C5", 1.0)])
def test_larger_conditioning_std_sits_on_the_format_floor(name, cond_std):
    """Record of what the HIP path does on the inputs the named workloads do NOT use because the format itself comes too
    close to the bar there (tests/golden/bf16_floor.txt: the float64 oracle with nothing but bf16 storage rounding costs
    2.3e-2 / 2.5e-2 on the 7-layer Flux-scale stage at conditioning std 0.5 / 1, 1.6e-2 on the SD3-scale stage at 1).
    The HIP path has to sit on that floor: the same typical (rms) error within 5 %, and a maximum error within a
    quarter of the floor's (two realisations of the same rounding noise, maximum over millions of outputs)."""
    floor_max, floor_rms = _golden_floor(name, cond_std)
    assert floor_max > TOL * 2 / 3               # the reason this input is not the named workload's
    if wl.CONFIGS[name]["seq_img"] > 8192:
        err, et, ek = _one_call(name, wl.CONFIGS[name]["n_patches"] - 1, False, cond_std=cond_std)
        rms = _LAST["rms"]
    else:
        err, rms = _last_patch_after_fill(wl.variant(wl.CONFIGS[name], cond_std=cond_std))
    _log(f"  {name} cond std {cond_std}: HIP max {err:.3e} rms {rms:.3e}; storage floor max {floor_max:.3e} rms {floor_rms:.3e}")
    assert err < 1.25 * floor_max
    assert rms < 1.05 * floor_rms


def _last_patch_after_fill(cfg):
    """The golden file's call for the workloads that are built per test: last patch, image only, synthetic stale buffer."""
    W, A = wl.make_weights(cfg), wl.make_activations(cfg)
    st = _pkg().Stage(cfg, W)
    orc = StageOracle(cfg, W)
    if cfg["kind"] == 1:
        st.kv_init(None, None, _f32(A["text"]).to(torch.bfloat16))
        orc.kv_init(None, text=A["text"])
    else:
        st.kv_init(None)
        orc.kv_init(None)
    fills = [wl.make_kv_fill(cfg, l) for l in range(cfg["n_layers"])]
    _refill(st, orc, cfg, fills)
    n, p = wl.patch_rows(cfg), cfg["n_patches"] - 1
    xp = A["x"][p * n:(p + 1) * n]
    y = st.patch_forward(_f32(xp), _f32(A["cond"]), p)
    torch.cuda.synchronize()
    ref = orc.patch_forward(xp, A["cond"], p)
    st.destroy()
    return _relerr(y, ref), _rmserr(y, ref)


def _golden_floor(name, cond_std):
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "bf16_floor.txt")
    for line in open(path):
        f = line.split()
        if len(f) >= 4 and not line.startswith("#") and f[0] == name and float(f[1]) == cond_std:
            return float(f[2]), float(f[3])
    raise KeyError((name, cond_std))
