"""Sampling-loop parity (GPU): N chained stage objects, M patches, S steps with the Euler update, against the CPU
pipeline oracle on the same seeded inputs.  Errors of consecutive steps add up, so the bar is the per-call bar
(1e-4 rms fp32, 2e-2 rms bf16) times the number of steps; every step's network output is checked too."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle.pf_pipeline import PipelineOracle, euler_update

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}


def _log(*a):
    print(*a, flush=True)


def _f32(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def _text_dev(cfg, A):
    if A["text"] is None:
        return None
    if cfg["kind"] == 1:
        return _f32(A["text"]).to(torch.bfloat16 if cfg["dtype"] == "bf16" else torch.float32)
    return _f32(A["text"])


def _relerr(got, ref):
    got = got.detach().double().cpu().numpy()
    return float(np.max(np.abs(got - ref)) / (np.sqrt(np.mean(ref ** 2)) + 1e-30))


def test_axpy_matches_update_rule():
    from paper_2405_14430_amd import pf_op_axpy
    rng = np.random.default_rng(5)
    for n in (0, 1, 255, 257, 300 * 192 + 3):
        x = rng.normal(size=n).astype(np.float32)
        e = rng.normal(size=n).astype(np.float32)
        _log("axpy n =", n)
        got = pf_op_axpy(_f32(x), _f32(e), -0.125)
        ref = euler_update(x, e, -0.125)
        assert got.shape == (n,)
        if n:
            assert np.max(np.abs(got.double().cpu().numpy() - ref)) <= 2.0 ** -23 * np.max(np.abs(ref))
    from paper_2405_14430_amd import pf_op_axpby
    xa, ea = rng.normal(size=777).astype(np.float32), rng.normal(size=777).astype(np.float32)
    got = pf_op_axpby(_f32(xa), _f32(ea), 0.75, -0.3)
    ref = 0.75 * xa.astype(np.float64) - 0.3 * ea.astype(np.float64)
    assert np.max(np.abs(got.double().cpu().numpy() - ref)) <= 2.0 ** -22 * np.max(np.abs(ref))
    x = _f32(rng.normal(size=1000).astype(np.float32))
    keep = x.clone()
    pf_op_axpy(x, x.clone(), 0.5, out=x)                 # in place
    assert torch.equal(x, keep * 1.5)


@pytest.mark.parametrize("name,N,S", [("K0f", 2, 3), ("K1f", 2, 3), ("K2f", 2, 3), ("K3f", 2, 3), ("K0f", 3, 2),
                                      ("C2s", 2, 3), ("C3s", 2, 3), ("C4s", 2, 2), ("K2n", 2, 2), ("C4n", 2, 2)])
def test_sampling_loop_matches_oracle(name, N, S):
    from paper_2405_14430_amd.pipeline import Pipeline
    cfg = wl.CONFIGS[name]
    W = wl.make_weights(cfg, n_layers=N * cfg["n_layers"])
    A = wl.make_activations(cfg)
    conds, dts = wl.make_sampling(cfg, S)
    _log("pipeline", name, "N", N, "M", cfg["n_patches"], "S", S)
    orc = PipelineOracle(cfg, wl.split_stages(W, N))
    ref, trace = orc.run(A["x"], conds, dts, warmup_steps=1, text=A["text"])

    pipe = Pipeline(cfg, wl.split_stages(W, N))
    text = _text_dev(cfg, A)
    x = _f32(A["x"]).clone()
    tol = TOL[cfg["dtype"]]
    try:
        for s in range(S):
            c = _f32(conds[s])
            eps = pipe.warmup_step(x, c, text) if s == 0 else pipe.pipelined_step(x, c, text)
            e = _relerr(eps, trace[s])
            _log("  step", s, "eps err", e)
            assert e < tol * (s + 1)
            from paper_2405_14430_amd import pf_op_axpy
            pf_op_axpy(x, eps, dts[s], out=x)
        assert _relerr(x, ref) < tol * S
        # the packaged loop gives the same bits as the step-by-step calls above
        x2 = pipe.run(_f32(A["x"]), [_f32(c) for c in conds], dts, warmup_steps=1, text=text)
        assert torch.equal(x2, x)
    finally:
        pipe.destroy()


@pytest.mark.parametrize("name,S", [("K0f", 3), ("K1f", 2), ("K3f", 2), ("C2s", 3), ("C3s", 2)])
def test_guided_sampling_loop_matches_oracle(name, S):
    """Classifier-free guidance: conditional and unconditional pass share every call (batch 2)."""
    from paper_2405_14430_amd.pipeline import CfgPipeline
    from oracle.pf_pipeline import CfgPipelineOracle
    cfg = wl.CONFIGS[name]
    ucfg = wl.variant(cfg, seed=cfg["seed"] + 100)
    N, scale = 2, 3.0
    W = wl.make_weights(cfg, n_layers=N * cfg["n_layers"])
    A, U = wl.make_activations(cfg), wl.make_activations(ucfg)
    conds_c, dts = wl.make_sampling(cfg, S)
    conds_u, _ = wl.make_sampling(ucfg, S)
    _log("guided pipeline", name, "S", S)
    ref, trace = CfgPipelineOracle(cfg, wl.split_stages(W, N)).run(A["x"], conds_c, conds_u, dts, scale, 1, A["text"], U["text"])
    pipe = CfgPipeline(cfg, wl.split_stages(W, N))
    text2 = None
    if A["text"] is not None:
        text2 = _f32(np.stack([A["text"], U["text"]], 0))
        if cfg["kind"] == 1:
            text2 = text2.to(torch.bfloat16 if cfg["dtype"] == "bf16" else torch.float32)
    conds2 = [_f32(np.stack([c, u], 0)) for c, u in zip(conds_c, conds_u)]
    tol = TOL[cfg["dtype"]] * (1.0 + 2.0 * (scale - 1.0))     # the guided eps amplifies the difference of two passes
    try:
        x = pipe.run(_f32(A["x"]), conds2, dts, scale, warmup_steps=1, text2=text2)
        torch.cuda.synchronize()
        e = _relerr(x, ref)
        _log("  final latent err", e)
        assert e < tol * S
    finally:
        pipe.destroy()


@pytest.mark.parametrize("i", list(range(10)))
def test_sampling_loop_random_configurations(i):
    """The sampling loop on drawn stage configurations (same generator as the random stage sweep), N = 2 or 3 stages,
    two or three steps, the first one synchronous."""
    from test_gpu_random_stages import _draw_config
    from paper_2405_14430_amd.pipeline import Pipeline
    cfg, _, rng = _draw_config(100 + i)
    cfg = wl.variant(cfg, txt_pre_only_last=0)            # a per-stage property; the loop builds every stage from one cfg
    N, S = int(rng.integers(2, 4)), int(rng.integers(2, 4))
    _log("random pipeline", i, {k: cfg[k] for k in ("kind", "dtype", "n_layers", "hidden", "head_dim", "seq_img", "n_patches",
                                                     "text_len", "qk_norm", "joint_rope")}, "N", N, "S", S)
    W = wl.make_weights(cfg, n_layers=N * cfg["n_layers"])
    A = wl.make_activations(cfg)
    conds, dts = wl.make_sampling(cfg, S)
    ref, trace = PipelineOracle(cfg, wl.split_stages(W, N)).run(A["x"], conds, dts, warmup_steps=1, text=A["text"])
    pipe = Pipeline(cfg, wl.split_stages(W, N))
    try:
        x = pipe.run(_f32(A["x"]), [_f32(c) for c in conds], dts, warmup_steps=1, text=_text_dev(cfg, A))
        torch.cuda.synchronize()
        assert _relerr(x, ref) < TOL[cfg["dtype"]] * S
    finally:
        pipe.destroy()
