"""Seeded random-shape sweeps of the single-operator entry points against the CPU oracle (GPU).

The fixed cases elsewhere pick the shapes the workloads use and the tile boundaries known to matter; here the
shapes are drawn (Philox, fixed keys) so that ragged tails, odd tile counts and splits that nobody thought of get
their turn: GEMM with both epilogues on every path, patch attention with every head size the bf16 kernels
specialise (and one they do not), key splits included."""
import math

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import pf_oracle as po

pytestmark = pytest.mark.gpu

F32, BF = torch.float32, torch.bfloat16


def _pkg():
    import paper_2405_14430_amd as pkg
    return pkg


def _rng(key):
    return np.random.Generator(np.random.Philox(key=key))


def _draw(rng, shape, dtype, std=1.0):
    a = rng.standard_normal(shape, dtype=np.float32) * np.float32(std)
    return wl.round_to_bf16(a) if dtype == BF else a


def _dev(a, dtype):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda().to(dtype)


def _close(got, ref, slack):
    """bf16 output: one bf16 rounding (2^-8 relative) of the fp64 value plus slack * rms; fp32 output: slack * rms."""
    g = got.detach().double().cpu().numpy()
    rms = np.sqrt(np.mean(ref ** 2)) + 1e-30
    bound = (2.0 ** -8) * np.abs(ref) * (1.0 if got.dtype == BF else 0.0) + slack * rms
    return bool(np.all(np.abs(g - ref) <= bound))


def _gemm_shapes(count, key):
    rng = _rng(key)
    out = []
    for _ in range(count):
        M = int(rng.integers(1, 700))
        N = int(rng.integers(1, 90)) * 8 if rng.random() < 0.7 else int(rng.integers(1, 700))
        K = int(rng.integers(1, 40)) * (64 if rng.random() < 0.6 else 8)
        out.append((M, N, K))
    return out


@pytest.mark.parametrize("dtype,path,slack", [(F32, 1, 2e-5), (BF, 1, 1e-3), (BF, 0, 1e-3)])
def test_gemm_random_shapes(dtype, path, slack):
    pkg = _pkg()
    for i, (M, N, K) in enumerate(_gemm_shapes(24, 20240 + path)):
        print("gemm random", dtype, path, M, N, K, flush=True)
        rng = _rng(1000 * i + M + N + K)
        A, W, b = _draw(rng, (M, K), dtype), _draw(rng, (N, K), dtype, 1 / math.sqrt(K)), _draw(rng, (N,), dtype)
        gate, R = _draw(rng, (N,), F32), _draw(rng, (M, N), F32)
        gf = int(rng.integers(0, N + 1)) // 8 * 8
        got = pkg.pf_op_gemm(_dev(A, dtype), _dev(W, dtype), _dev(b, dtype), epilogue=0, gelu_from=gf, path=path)
        x, xb = pkg.pf_op_gemm(_dev(A, dtype), _dev(W, dtype), _dev(b, dtype), epilogue=1, gate=_dev(gate, F32),
                               R=_dev(R, F32), want_copy=True, path=path)
        torch.cuda.synchronize()
        lin = po.linear(A, W, b)
        ref = lin.copy()
        ref[:, gf:] = po.gelu(ref[:, gf:], True)
        assert _close(got, ref, slack), (M, N, K, "store")
        assert _close(x, R.astype(np.float64) + gate.astype(np.float64) * lin, slack), (M, N, K, "residual")
        assert torch.equal(xb, x.to(dtype)), (M, N, K, "copy")


def _kv_buffers(k, v, H, dh, dtype):
    rows = k.shape[0]
    Lp = (rows + 127) // 128 * 128
    K = torch.zeros(H, Lp, dh, dtype=dtype, device="cuda")
    Vt = torch.zeros(H, dh, Lp, dtype=dtype, device="cuda")
    K[:, :rows] = _dev(k, dtype).view(rows, H, dh).transpose(0, 1)
    Vt[:, :, :rows] = _dev(v, dtype).view(rows, H, dh).permute(1, 2, 0)
    return K, Vt, Lp


@pytest.mark.parametrize("dtype,path,slack", [(F32, 1, 1e-4), (BF, 1, 1e-2), (BF, 0, 1e-2)])
def test_attention_random_shapes(dtype, path, slack):
    pkg = _pkg()
    rng0 = _rng(777 + path)
    for i in range(20):
        dh = int(rng0.choice([64, 72, 128, 40]))
        H = int(rng0.integers(1, 4))
        nq = int(rng0.integers(1, 1500)) if rng0.random() < 0.5 else int(rng0.integers(1, 200))
        Lkv = int(rng0.integers(1, 2200))
        tiles = (Lkv + 63) // 64
        splits = int(rng0.integers(1, min(tiles, 9) + 1))
        gain = float(rng0.choice([1.0, 4.0]))
        print("attention random", dtype, path, H, dh, nq, Lkv, splits, gain, flush=True)
        rng = _rng(5000 + i)
        q, k, v = _draw(rng, (nq, H * dh), dtype, gain), _draw(rng, (Lkv, H * dh), dtype), _draw(rng, (Lkv, H * dh), dtype)
        K, Vt, Lp = _kv_buffers(k, v, H, dh, dtype)
        got = pkg.pf_op_attention(_dev(q, dtype), K, Vt, Lkv, Lp, H, dh, splits=splits, path=path)
        torch.cuda.synchronize()
        assert _close(got, po.attention(q, k, v, H), slack), (H, dh, nq, Lkv, splits, gain)
