"""Batched patch calls (B images per call, e.g. the conditional and unconditional image of classifier-free guidance)
through the C boundary against B independent CPU oracles that share the weights: warm-up pass, a sweep over the patches
(text rows ride with patch 0 for the joint kinds), and every image's K/V buffers.  Same bars as the single-image
tests."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle.pf_oracle import StageOracle

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}


def _log(*a):
    print(*a, flush=True)


def _f32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def _relerr(got, ref):
    got = got.detach().double().cpu().numpy()
    return float(np.max(np.abs(got - ref)) / (np.sqrt(np.mean(ref ** 2)) + 1e-30))


def _kv_close(got, ref, dtype):
    rms = np.sqrt(np.mean(ref ** 2)) + 1e-30
    if dtype == "f32":
        return float(np.max(np.abs(got - ref))) < 1e-4 * rms
    return bool(np.all(np.abs(got - ref) <= 2.0 ** -8 * np.abs(ref) + 2e-2 * rms))


def _natural(Kview):
    r, H, dh = Kview.shape
    return Kview.double().cpu().numpy().reshape(r, H * dh)


def _images(cfg, B):
    """Activations of B different images (own latent, conditioning and text each)."""
    return [wl.make_activations(wl.variant(cfg, seed=cfg["seed"] + 100 * b)) for b in range(B)]


def _stack(acts, key):
    return np.stack([a[key] for a in acts], axis=0)


CASES = [("K0f", 2, 0), ("K1f", 2, 0), ("K2f", 2, 0), ("K3f", 2, 0), ("K1f", 3, 0),
         ("C2s", 2, 0), ("C2x", 2, 0), ("C3p", 2, 0), ("C3s", 2, 0), ("C4s", 2, 0), ("C5s", 2, 0), ("C2s", 2, 1), ("C3s", 3, 0),
         ("K2n", 2, 0), ("C3n", 2, 0), ("C4n", 2, 0), ("C3r", 2, 0)]


@pytest.mark.parametrize("name,B,path", CASES)
def test_batched_sweep_matches_independent_oracles(name, B, path):
    from paper_2405_14430_amd import Stage
    cfg = wl.CONFIGS[name]
    tol = TOL[cfg["dtype"]]
    W = wl.make_weights(cfg)
    acts = _images(cfg, B)
    kind, joint = cfg["kind"], cfg["kind"] in (2, 3)
    _log("batched sweep", name, "B", B, "path", path)
    st = Stage(dict(cfg, batch=B), W, kernel_path=path)
    orcs = [StageOracle(cfg, W) for _ in range(B)]
    cond = _f32(_stack(acts, "cond"))
    text = None
    if kind == 1:
        text = _f32(_stack(acts, "text")).to(st.dt)
    elif joint:
        text = _f32(_stack(acts, "text"))

    y0, t0 = st.kv_init(_f32(_stack(acts, "x_prev")), cond, text, want_output=True)
    torch.cuda.synchronize()
    for b in range(B):
        ref0, reft0 = orcs[b].kv_init(acts[b]["x_prev"], acts[b]["cond"], text=acts[b]["text"])
        assert _relerr(y0[b], ref0) < tol
        if joint:
            assert _relerr(t0[b], reft0) < tol

    n = wl.patch_rows(cfg)
    for p in range(cfg["n_patches"]):
        xp = _f32(np.stack([a["x"][p * n:(p + 1) * n] for a in acts], axis=0))
        if joint and p == 0:
            y, yt = st.patch_forward(xp, cond, p, text=text)
        else:
            y, yt = st.patch_forward(xp, cond, p), None
        torch.cuda.synchronize()
        for b in range(B):
            a = acts[b]
            if yt is not None:
                ref, reft = orcs[b].patch_forward(a["x"][p * n:(p + 1) * n], a["cond"], p, text=a["text"])
                assert _relerr(yt[b], reft) < tol
            else:
                ref = orcs[b].patch_forward(a["x"][p * n:(p + 1) * n], a["cond"], p)
            err = _relerr(y[b], ref)
            _log(f"  patch {p} image {b}: err {err:.3e}")
            assert err < tol
    for l in range(len(W)):
        for b in range(B):
            K, V, view = st.kv_view(l, image=b)
            assert view.rows == wl.kv_rows(cfg)
            assert _kv_close(_natural(K), orcs[b].kbuf[l], cfg["dtype"])
            assert _kv_close(_natural(V), orcs[b].vbuf[l], cfg["dtype"])
            if kind == 1:
                Kc, Vc, _ = st.xattn_kv_view(l, image=b)
                assert _kv_close(_natural(Kc), orcs[b].kc[l], cfg["dtype"])
                assert _kv_close(_natural(Vc), orcs[b].vc[l], cfg["dtype"])
    st.destroy()


@pytest.mark.parametrize("name", ["K2f", "C4s"])
def test_batched_zero_init_image_only_calls(name):
    """App. B start (zero buffers) and image-only calls out of order: every image still matches its own oracle."""
    from paper_2405_14430_amd import Stage
    cfg = wl.CONFIGS[name]
    tol, B = TOL[cfg["dtype"]], 2
    W = wl.make_weights(cfg)
    acts = _images(cfg, B)
    st = Stage(dict(cfg, batch=B), W)
    orcs = [StageOracle(cfg, W) for _ in range(B)]
    st.kv_init(None)
    for o in orcs:
        o.kv_init(None)
    cond = _f32(_stack(acts, "cond"))
    n = wl.patch_rows(cfg)
    for p in (cfg["n_patches"] - 1, 0, 1):
        xp = _f32(np.stack([a["x"][p * n:(p + 1) * n] for a in acts], axis=0))
        y = st.patch_forward(xp, cond, p)
        torch.cuda.synchronize()
        for b in range(B):
            ref = orcs[b].patch_forward(acts[b]["x"][p * n:(p + 1) * n], acts[b]["cond"], p)
            assert _relerr(y[b], ref) < tol


def test_batch_of_one_field_values_agree():
    """batch = 0 and batch = 1 both mean one image and give the same bits."""
    from paper_2405_14430_amd import Stage
    cfg = wl.CONFIGS["C2s"]
    W, A = wl.make_weights(cfg), wl.make_activations(cfg)
    outs = []
    for bval in (0, 1):
        st = Stage(dict(cfg, batch=bval), W)
        cond = _f32(A["cond"])
        st.kv_init(_f32(A["x_prev"]), cond, _f32(A["text"]).to(st.dt))
        n = wl.patch_rows(cfg)
        outs.append(st.patch_forward(_f32(A["x"][n:2 * n]), cond, 1).clone())
        st.destroy()
    assert torch.equal(outs[0], outs[1])
