"""The entry point that allocates nothing (pf_op_attention_static): its split partial results live in the library's
static device array instead of a workspace argument.  Checked against pf_op_attention (same kernels, same splits) and
against the CPU oracle, on two calls in a row, the second with a smaller input, so that the second call runs over the
first call's leftovers in the shared array."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import pf_oracle as po

pytestmark = pytest.mark.gpu
BF, F32 = torch.bfloat16, torch.float32
TOL = {F32: 1e-4, BF: 2e-2}


def _pkg():
    import paper_2405_14430_amd as pkg
    return pkg


def _draw(rng, shape, dtype, std=1.0):
    a = rng.standard_normal(shape, dtype=np.float32) * np.float32(std)
    return wl.round_to_bf16(a) if dtype == BF else a


def _dev(a, dtype):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda().to(dtype)


def _kv(k, v, H, dh, dtype):
    rows = k.shape[0]
    Lp = (rows + 127) // 128 * 128
    K = torch.zeros(H, Lp, dh, dtype=dtype, device="cuda")
    Vt = torch.zeros(H, dh, Lp, dtype=dtype, device="cuda")
    K[:, :rows] = _dev(k, dtype).view(rows, H, dh).transpose(0, 1)
    Vt[:, :, :rows] = _dev(v, dtype).view(rows, H, dh).permute(1, 2, 0)
    return K, Vt, Lp


def _within_bar(got, ref, dtype):
    """fp32: max|err| <= 1e-4 rms.  bf16: the output is STORED in bf16, so an element may be off by one storage
    rounding of its own value (2^-8 relative: a 5-sigma element alone is 2e-2 rms) plus half the 2e-2 rms bar for the
    arithmetic in front of it (bf16 softmax weights, fp32 accumulation)."""
    g = got.detach().double().cpu().numpy()
    rms = np.sqrt(np.mean(ref ** 2)) + 1e-30
    if dtype == F32:
        return float(np.max(np.abs(g - ref))) <= TOL[F32] * rms
    return bool(np.all(np.abs(g - ref) <= 2.0 ** -8 * np.abs(ref) + 0.5 * TOL[BF] * rms))


@pytest.mark.parametrize("dtype,path,dh", [(BF, 0, 72), (BF, 0, 128), (BF, 0, 40), (F32, 1, 64)])
def test_static_scratch_attention_matches_workspace_attention_twice(dtype, path, dh):
    pkg = _pkg()
    H = 3
    # first call: larger, 6 splits; second call: fewer queries, keys and splits (its partials cover a prefix of what
    # the first call left in the array, with a different layout)
    for nq, Lkv, splits in ((300, 1500, 6), (77, 700, 3)):
        print("static attention", dtype, path, dh, nq, Lkv, splits, flush=True)
        rng = np.random.Generator(np.random.Philox(key=dh * 1000 + nq))
        q, k, v = _draw(rng, (nq, H * dh), dtype), _draw(rng, (Lkv, H * dh), dtype), _draw(rng, (Lkv, H * dh), dtype)
        K, Vt, Lp = _kv(k, v, H, dh, dtype)
        qd = _dev(q, dtype)
        out = torch.full((nq, H * dh), float("nan"), dtype=dtype, device="cuda")
        pkg.pf_op_attention_static(qd, K, Vt, Lkv, Lp, H, dh, out, splits=splits, path=path)
        ref_dev = pkg.pf_op_attention(qd, K, Vt, Lkv, Lp, H, dh, splits=splits, path=path)
        torch.cuda.synchronize()
        ref = po.attention(q, k, v, H)
        assert _within_bar(out, ref, dtype)
        assert _within_bar(ref_dev, ref, dtype)
        assert torch.equal(out, ref_dev)          # same kernels, same split: same bits


def test_static_scratch_attention_rejects_what_does_not_fit():
    pkg = _pkg()
    lib = pkg.load_library()
    cap = lib.pf_static_scratch_bytes()
    assert cap == 32 << 20
    H, dh, nq, Lkv, splits = 16, 72, 4096, 4096, 8          # 151 MB of partials
    assert lib.pf_op_attention_ws_bytes(nq, H, dh, splits) > cap
    q = torch.zeros(nq, H * dh, dtype=BF, device="cuda")
    K = torch.zeros(H, Lkv, dh, dtype=BF, device="cuda")
    Vt = torch.zeros(H, dh, Lkv, dtype=BF, device="cuda")
    out = torch.zeros_like(q)
    with pytest.raises(pkg.PfError) as e:
        pkg.pf_op_attention_static(q, K, Vt, Lkv, Lkv, H, dh, out, splits=splits)
    assert e.value.status == -7 and "static scratch" in str(e.value)
    # one split needs no scratch at all and passes whatever the size
    pkg.pf_op_attention_static(q, K, Vt, Lkv, Lkv, H, dh, out, splits=1)
    torch.cuda.synchronize()
