"""Kernel-level parity (GPU): every operator of the path, called through the C boundary, against the matching
function of the CPU oracle on the same seeded inputs.  Shapes span several tiles and ragged tails."""
import math

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import pf_oracle as po

pytestmark = pytest.mark.gpu

BF, F32 = torch.bfloat16, torch.float32
TOL = {F32: 1e-4, BF: 2e-2}     # max|err| / rms(ref): the bars of the stage, reused per operator


def _pkg():
    import paper_2405_14430_amd as pkg
    return pkg


def _rng(seed):
    return np.random.Generator(np.random.Philox(key=seed))


def _draw(rng, shape, dtype, std=1.0):
    a = (rng.standard_normal(shape, dtype=np.float32) * np.float32(std))
    return wl.round_to_bf16(a) if dtype == BF else a


def _dev(a, dtype):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda().to(dtype)


def _relerr(got, ref):
    got = got.detach().double().cpu().numpy()
    return float(np.max(np.abs(got - ref)) / (np.sqrt(np.mean(ref ** 2)) + 1e-30))


def _log(*a):
    print(*a, flush=True)


def _close(got, ref, dtype, slack=1e-3):
    """fp32: max|err| <= 2e-5 rms.  bf16 output: each element within one bf16 rounding (2^-8 relative) of the fp64
    value plus `slack` * rms for the fp32-accumulated bf16 operands."""
    g = got.detach().double().cpu().numpy()
    rms = np.sqrt(np.mean(ref ** 2)) + 1e-30
    if dtype == F32 and got.dtype == F32:
        return float(np.max(np.abs(g - ref))) <= 2e-5 * rms
    bound = (2.0 ** -8) * np.abs(ref) * (1.0 if got.dtype == BF else 0.0) + slack * rms
    return bool(np.all(np.abs(g - ref) <= bound))


@pytest.mark.parametrize("dtype", [F32, BF])
@pytest.mark.parametrize("rows,d", [(67, 384), (130, 1152), (5, 3072), (33, 200), (9, 8192)])
def test_ln_modulate(dtype, rows, d):
    _log("ln_modulate", dtype, rows, d)
    rng = _rng(rows * 10007 + d)
    x = _draw(rng, (rows, d), F32) * 2 + 0.5
    sh, sc = _draw(rng, (d,), F32), _draw(rng, (d,), F32)
    got = _pkg().pf_op_ln_modulate(_dev(x, F32), _dev(sh, F32), _dev(sc, F32), 1e-6, dtype)
    torch.cuda.synchronize()
    assert _close(got, po.ln_modulate(x, sh, sc, 1e-6), dtype, 1e-5)
    plain = _pkg().pf_op_ln_modulate(_dev(x, F32), None, None, 1e-6, dtype, normalize=False)
    torch.cuda.synchronize()
    assert torch.equal(plain, _dev(x, F32).to(dtype))


@pytest.mark.parametrize("dtype", [F32, BF])
@pytest.mark.parametrize("d,out", [(1152, 6 * 1152 + 8), (200, 37), (64, 3), (1536, 2 * 1536 + 1)])
def test_modulation(dtype, d, out):
    """Output widths that are no multiple of the eight rows a wave streams side by side, or of a block's 32."""
    rng = _rng(5 + d + out)
    w, b, c = _draw(rng, (out, d), dtype, 0.02), _draw(rng, (out,), dtype, 0.02), _draw(rng, (d,), F32)
    got = _pkg().pf_op_modulation(_dev(w, dtype), _dev(b, dtype), _dev(c, F32))
    torch.cuda.synchronize()
    assert _relerr(got, po.linear(po.silu(c), w, b)) < 1e-5
    table, c6 = _draw(rng, (6, d), dtype, 0.02), _draw(rng, (6 * d,), F32)
    got = _pkg().pf_op_modulation(_dev(table, dtype), None, _dev(c6, F32), table_mode=True)
    torch.cuda.synchronize()
    assert _relerr(got, table.reshape(-1).astype(np.float64) + c6) < 1e-6


GEMM_SHAPES = [(67, 200, 136), (512, 3456, 1152), (130, 1152, 4608), (1, 72, 8), (300, 264, 72), (257, 130, 192),
               (2100, 1000, 640), (4100, 2050, 128), (33, 70, 64)]


@pytest.mark.parametrize("dtype,path", [(F32, 1), (BF, 1), (BF, 0)])
@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
def test_gemm_store_epilogue_with_gelu_columns(dtype, path, M, N, K):
    _log("gemm/store", dtype, path, M, N, K)
    rng = _rng(M * 31 + N * 7 + K)
    A, W, b = _draw(rng, (M, K), dtype), _draw(rng, (N, K), dtype, 1 / math.sqrt(K)), _draw(rng, (N,), dtype)
    gf = (N // 3) // 8 * 8
    got = _pkg().pf_op_gemm(_dev(A, dtype), _dev(W, dtype), _dev(b, dtype), epilogue=0, gelu_from=gf, path=path)
    torch.cuda.synchronize()
    ref = po.linear(A, W, b)
    ref[:, gf:] = po.gelu(ref[:, gf:], True)
    assert _close(got, ref, dtype)


@pytest.mark.parametrize("dtype,path", [(F32, 1), (BF, 1), (BF, 0)])
@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
def test_gemm_gated_residual_epilogue(dtype, path, M, N, K):
    _log("gemm/residual", dtype, path, M, N, K)
    rng = _rng(M * 13 + N * 5 + K + 1)
    A, W, b = _draw(rng, (M, K), dtype), _draw(rng, (N, K), dtype, 1 / math.sqrt(K)), _draw(rng, (N,), dtype)
    gate, R = _draw(rng, (N,), F32), _draw(rng, (M, N), F32)
    x, xb = _pkg().pf_op_gemm(_dev(A, dtype), _dev(W, dtype), _dev(b, dtype), epilogue=1, gate=_dev(gate, F32),
                              R=_dev(R, F32), want_copy=True, path=path)
    torch.cuda.synchronize()
    ref = R.astype(np.float64) + gate.astype(np.float64) * po.linear(A, W, b)
    assert x.dtype == F32 and _close(x, ref, dtype)
    assert torch.equal(xb, x.to(dtype))                      # the rounded copy is the rounding of what was stored
    # erf GELU flavour and gate = None (plain residual)
    x2, _ = _pkg().pf_op_gemm(_dev(A, dtype), _dev(W, dtype), _dev(b, dtype), epilogue=1, R=_dev(R, F32), path=path)
    torch.cuda.synchronize()
    assert _close(x2, R.astype(np.float64) + po.linear(A, W, b), dtype)


@pytest.mark.parametrize("tile_id", list(range(1, 13)))
def test_gemm_every_tile_configuration(tile_id):
    """Each bf16 tile configuration the heuristic chooses from, pinned for the one launch through pf_op_gemm_tile, on a
    shape with ragged M and N, for both epilogues."""
    pkg = _pkg()
    lib = pkg.load_library()
    assert lib.pf_gemm_tile_count() == 12
    M, N, K = 777, 650, 320
    rng = _rng(4242 + tile_id)
    A, W, b = _draw(rng, (M, K), BF), _draw(rng, (N, K), BF, 1 / math.sqrt(K)), _draw(rng, (N,), BF)
    gate, R = _draw(rng, (N,), F32), _draw(rng, (M, N), F32)
    got = pkg.pf_op_gemm(_dev(A, BF), _dev(W, BF), _dev(b, BF), epilogue=0, gelu_from=320, tile=tile_id)
    x, xb = pkg.pf_op_gemm(_dev(A, BF), _dev(W, BF), _dev(b, BF), epilogue=1, gate=_dev(gate, F32), R=_dev(R, F32),
                           want_copy=True, tile=tile_id)
    torch.cuda.synchronize()
    ref = po.linear(A, W, b)
    refx = R.astype(np.float64) + gate.astype(np.float64) * ref
    ref[:, 320:] = po.gelu(ref[:, 320:], True)
    assert _close(got, ref, BF) and _close(x, refx, BF) and torch.equal(xb, x.to(BF))


@pytest.mark.parametrize("tile_id", [7, 8, 3, 6, 12])   # 64x64 four / three stages, 256x128 three stages, wave-split-K, 128x192 three stages
@pytest.mark.parametrize("K", [64, 128, 192])
def test_gemm_rings_on_short_k(tile_id, K):
    """Fewer K tiles than ring stages: prologue and drain only."""
    pkg = _pkg()
    M, N = 130, 200
    rng = _rng(999 + tile_id + K)
    A, W, b = _draw(rng, (M, K), BF), _draw(rng, (N, K), BF, 1 / math.sqrt(K)), _draw(rng, (N,), BF)
    got = pkg.pf_op_gemm(_dev(A, BF), _dev(W, BF), _dev(b, BF), epilogue=0, tile=tile_id)
    torch.cuda.synchronize()
    assert _close(got, po.linear(A, W, b), BF)


def test_gemm_erf_gelu():
    rng = _rng(77)
    A, W, b = _draw(rng, (40, 64), F32), _draw(rng, (48, 64), F32, 0.2), _draw(rng, (48,), F32)
    got = _pkg().pf_op_gemm(_dev(A, F32), _dev(W, F32), _dev(b, F32), epilogue=0, gelu_from=0, gelu_tanh=0, path=1)
    torch.cuda.synchronize()
    assert _relerr(got, po.gelu(po.linear(A, W, b), False)) < 2e-5


def _kv_buffers(k, v, H, dh, dtype, sentinel=None):
    """Natural [rows, H*dh] arrays -> device K [H][Lp][dh] and V^T [H][dh][Lp] (padding rows zero)."""
    rows = k.shape[0]
    Lp = (rows + 127) // 128 * 128
    K = torch.zeros(H, Lp, dh, dtype=dtype, device="cuda")
    Vt = torch.zeros(H, dh, Lp, dtype=dtype, device="cuda")
    K[:, :rows] = _dev(k, dtype).view(rows, H, dh).transpose(0, 1)
    Vt[:, :, :rows] = _dev(v, dtype).view(rows, H, dh).permute(1, 2, 0)
    return K, Vt, Lp


@pytest.mark.parametrize("dtype", [F32, BF])
@pytest.mark.parametrize("H,dh,rows,row0,Lp", [(4, 72, 150, 37, 384), (3, 64, 64, 0, 128), (2, 128, 70, 186, 256)])
def test_kv_scatter_positions_bit_exact(dtype, H, dh, rows, row0, Lp):
    """Fresh rows land at exactly rows [row0, row0+rows) of K and V^T, bit for bit; every other element of the
    buffers keeps its bits (PipeFusion Sec. 3.3: the rest of the buffer stays one step stale)."""
    _log("kv_scatter", dtype, H, dh, rows, row0, Lp)
    d = H * dh
    rng = _rng(H * 1000 + rows)
    qkv = _dev(_draw(rng, (rows, 3 * d), dtype), dtype)
    idt = torch.int16 if dtype == BF else torch.int32
    K = torch.randint(-30000, 30000, (H, Lp, dh), dtype=idt, device="cuda").view(dtype)
    Vt = torch.randint(-30000, 30000, (H, dh, Lp), dtype=idt, device="cuda").view(dtype)
    K0, V0, q0 = K.clone(), Vt.clone(), qkv.clone()
    _pkg().pf_op_kv_scatter(qkv, K, Vt, Lp, H, dh, row0)
    torch.cuda.synchronize()
    assert torch.equal(qkv.view(idt), q0.view(idt))          # without RoPE the projections are not touched
    expK, expV = K0.clone(), V0.clone()
    expK[:, row0:row0 + rows] = qkv[:, d:2 * d].reshape(rows, H, dh).transpose(0, 1)
    expV[:, :, row0:row0 + rows] = qkv[:, 2 * d:].reshape(rows, H, dh).permute(1, 2, 0)
    assert torch.equal(K.view(idt), expK.view(idt))
    assert torch.equal(Vt.view(idt), expV.view(idt))


@pytest.mark.parametrize("dtype", [F32, BF])
def test_kv_scatter_rope(dtype):
    H, dh, rows, row0, Lp, gw, tok0 = 2, 128, 75, 40, 256, 17, 91
    d = H * dh
    rng = _rng(99)
    qkv_np = _draw(rng, (rows, 3 * d), dtype)
    qkv = _dev(qkv_np, dtype)
    K = torch.zeros(H, Lp, dh, dtype=dtype, device="cuda")
    Vt = torch.zeros(H, dh, Lp, dtype=dtype, device="cuda")
    _pkg().pf_op_kv_scatter(qkv, K, Vt, Lp, H, dh, row0, rope=True, tok0=tok0, grid_w=gw, theta=1e4)
    torch.cuda.synchronize()
    toks = np.arange(tok0, tok0 + rows)
    ang = po.rope_angles(toks // gw, toks % gw, dh, 1e4)
    assert _close(qkv[:, :d], po.rope_apply(qkv_np[:, :d], ang, H), dtype, 1e-4)
    assert _close(qkv[:, d:2 * d], po.rope_apply(qkv_np[:, d:2 * d], ang, H), dtype, 1e-4)
    assert torch.equal(qkv[:, 2 * d:], _dev(qkv_np[:, 2 * d:], dtype))
    # the buffer holds exactly the rotated keys left in qkv, and v untouched
    assert torch.equal(K[:, row0:row0 + rows], qkv[:, d:2 * d].reshape(rows, H, dh).transpose(0, 1))
    assert torch.equal(Vt[:, :, row0:row0 + rows], qkv[:, 2 * d:].reshape(rows, H, dh).permute(1, 2, 0))
    # text rows (tok0 < 0) are not rotated
    qkv2 = _dev(qkv_np, dtype)
    _pkg().pf_op_kv_scatter(qkv2, K, Vt, Lp, H, dh, 0, rope=True, tok0=-1, grid_w=gw)
    torch.cuda.synchronize()
    assert torch.equal(qkv2, _dev(qkv_np, dtype))


@pytest.mark.parametrize("dtype", [F32, BF])
@pytest.mark.parametrize("H,dh,rope", [(3, 64, False), (2, 128, True), (5, 32, True)])
def test_kv_scatter_qk_rmsnorm(dtype, H, dh, rope):
    """q and k are RMS-normalised per head (then rotated) in place; K in the buffer is exactly what qkv then holds."""
    rows, row0, Lp, gw, tok0 = 77, 24, 128, 13, 5
    d = H * dh
    rng = _rng(123 + dh)
    qkv_np = _draw(rng, (rows, 3 * d), dtype, 3.0)
    wq, wk = _draw(rng, (dh,), dtype) * 0.25 + 1.0, _draw(rng, (dh,), dtype) * 0.25 + 1.0
    wq, wk = wl.round_to_bf16(wq) if dtype == BF else wq, wl.round_to_bf16(wk) if dtype == BF else wk
    qkv = _dev(qkv_np, dtype)
    K = torch.zeros(H, Lp, dh, dtype=dtype, device="cuda")
    Vt = torch.zeros(H, dh, Lp, dtype=dtype, device="cuda")
    _pkg().pf_op_kv_scatter(qkv, K, Vt, Lp, H, dh, row0, rope=rope, tok0=tok0, grid_w=gw, theta=1e4,
                            q_norm_w=_dev(wq, dtype), k_norm_w=_dev(wk, dtype), norm_eps=1e-6)
    torch.cuda.synchronize()
    qn = po.rms_norm_heads(qkv_np[:, :d], wq, H, 1e-6)
    kn = po.rms_norm_heads(qkv_np[:, d:2 * d], wk, H, 1e-6)
    if rope:
        toks = np.arange(tok0, tok0 + rows)
        ang = po.rope_angles(toks // gw, toks % gw, dh, 1e-4 * 0 + 1e4)
        qn, kn = po.rope_apply(qn, ang, H), po.rope_apply(kn, ang, H)
    assert _close(qkv[:, :d], qn, dtype, 1e-4) and _close(qkv[:, d:2 * d], kn, dtype, 1e-4)
    assert torch.equal(qkv[:, 2 * d:], _dev(qkv_np[:, 2 * d:], dtype))
    assert torch.equal(K[:, row0:row0 + rows], qkv[:, d:2 * d].reshape(rows, H, dh).transpose(0, 1))
    assert torch.equal(Vt[:, :, row0:row0 + rows], qkv[:, 2 * d:].reshape(rows, H, dh).permute(1, 2, 0))
    assert not bool(K[:, :row0].any()) and not bool(K[:, row0 + rows:].any())


ATTN_CASES = [  # H, dh, nq, Lkv, splits, gain (the last two: more splits than the combine kernel takes in one group,
    # and more splits than key tiles, so some splits see no key at all)
    (2, 64, 70, 333, 1, 1.0), (3, 72, 200, 1000, 3, 1.0), (2, 128, 130, 515, 2, 1.0), (2, 40, 33, 120, 1, 1.0),
    (2, 72, 100, 2100, 12, 4.0), (1, 64, 40, 700, 16, 1.0),
    (2, 72, 129, 4096, 4, 8.0), (1, 128, 64, 700, 5, 8.0), (4, 64, 256, 64, 1, 1.0), (2, 96, 31, 257, 1, 1.0),
]


@pytest.mark.parametrize("dtype,path", [(F32, 1), (BF, 1), (BF, 0)])
@pytest.mark.parametrize("H,dh,nq,Lkv,splits,gain", ATTN_CASES)
def test_attention(dtype, path, H, dh, nq, Lkv, splits, gain):
    """Patch queries over a full K/V buffer; gain > 1 peaks the softmax so the running-maximum rescale matters."""
    _log("attention", dtype, path, H, dh, nq, Lkv, splits, gain)
    d = H * dh
    rng = _rng(H * 100003 + dh * 1009 + nq * 13 + Lkv)
    q, k, v = _draw(rng, (nq, d), dtype, gain), _draw(rng, (Lkv, d), dtype), _draw(rng, (Lkv, d), dtype)
    K, Vt, Lp = _kv_buffers(k, v, H, dh, dtype)
    got = _pkg().pf_op_attention(_dev(q, dtype), K, Vt, Lkv, Lp, H, dh, splits=splits, path=path)
    torch.cuda.synchronize()
    assert _relerr(got, po.attention(q, k, v, H)) < TOL[dtype]


@pytest.mark.parametrize("dh", [64, 72, 128])
@pytest.mark.parametrize("nq,Lkv,splits,gain", [(1030, 50, 1, 1.0), (1024, 128, 1, 1.0), (1100, 190, 1, 4.0), (1281, 256, 1, 1.0),
                                                (1030, 300, 1, 1.0), (1030, 700, 1, 4.0), (1100, 1300, 3, 1.0),
                                                (1025, 2000, 2, 8.0)])
def test_attention_256_query_workgroups(dh, nq, Lkv, splits, gain):
    """Launches of at least 1024 query rows take the 8-wave kernel (256 queries per workgroup, four-stage ring, half of
    the waves on the rotated schedule): key-tile counts of every residue mod 4, ragged query and key tails, key splits."""
    _log("attention wide", dh, nq, Lkv, splits, gain)
    H = 2
    rng = _rng(dh * 1009 + nq * 13 + Lkv)
    q, k, v = _draw(rng, (nq, H * dh), BF, gain), _draw(rng, (Lkv, H * dh), BF), _draw(rng, (Lkv, H * dh), BF)
    K, Vt, Lp = _kv_buffers(k, v, H, dh, BF)
    got = _pkg().pf_op_attention(_dev(q, BF), K, Vt, Lkv, Lp, H, dh, splits=splits)
    torch.cuda.synchronize()
    assert _pkg().load_library().pf_attention_kernel_name(1, 0, dh, nq, 0).decode().split("<")[1].split(",")[3].rstrip(">") == "8"
    # 10^5 outputs stored in bf16: the storage rounding of a 4.5-sigma element alone is 2^-8 * 4.5 = 1.8e-2 rms, so the
    # bar here is one bf16 rounding of the value plus half the 2e-2 rms bar for the arithmetic
    assert _close(got, po.attention(q, k, v, H), BF, slack=1e-2)


def _attention_error_over_bar(got, q, k, v, H):
    """Largest element error of a bf16 attention output as a fraction of a bar derived from the arithmetic: the stored
    bf16 value is within 2^-9 of what was computed, twice over when key splits pass through fp16 partial rows
    (2^-8 |ref| covers both); every softmax weight reaches the matrix unit rounded to bf16 (2^-9 relative) and the
    denominator sums the same rounded or unrounded weights, so the weighted mean moves by at most
    2^-8 sum_j p_ij |v_jc| - the attention of |v|, which for peaked rows is of the size of the values, not of the
    output's rms; 2e-3 rms for the fp32 accumulation."""
    ref = po.attention(q, k, v, H)
    ref_abs = po.attention(q, k, np.abs(v), H)
    g = got.double().cpu().numpy()
    rms = np.sqrt(np.mean(ref ** 2))
    return float((np.abs(g - ref) / (2.0 ** -8 * np.abs(ref) + 2.0 ** -8 * ref_abs + 2e-3 * rms)).max())


@pytest.mark.parametrize("dh", [64, 72, 128])
@pytest.mark.parametrize("nq,Lkv,splits", [(200, 900, 1), (1100, 1500, 1), (1030, 2100, 3)])
@pytest.mark.parametrize("pattern", ["random", "rising", "falling", "late_spike", "huge_spike"])
def test_attention_prescaled_queries_reference_moves(dh, nq, Lkv, splits, pattern):
    """The kernels a stage launches take queries that already carry log2(e) / sqrt(dh) and form the softmax weights
    against a reference exponent that only moves when the weights say so.  Score patterns that make it move often
    (scores rising along the keys), never (falling), once and late (one key far above the rest), and by more than the
    exponent range of a float (a key whose score is hundreds of powers of two above the first tile's)."""
    _log("attention prescaled", dh, nq, Lkv, splits, pattern)
    H = 2
    rng = _rng(dh * 7919 + nq * 31 + Lkv + len(pattern))
    q, k, v = _draw(rng, (nq, H * dh), BF), _draw(rng, (Lkv, H * dh), BF), _draw(rng, (Lkv, H * dh), BF)
    if pattern in ("rising", "falling"):
        # a common direction u in every head: q.u > 0 for every query, k.u a ramp over the keys
        u = rng.standard_normal(dh).astype(np.float32)
        u /= np.linalg.norm(u)
        ramp = np.linspace(0.0, 6.0, Lkv, dtype=np.float32) * np.sqrt(dh)
        if pattern == "falling":
            ramp = ramp[::-1]
        for h in range(H):
            k[:, h * dh:(h + 1) * dh] += ramp[:, None] * u[None, :]
            q[:, h * dh:(h + 1) * dh] += 2.0 * u[None, :]
        k = wl.round_to_bf16(k)
        q = wl.round_to_bf16(q)
    elif pattern in ("late_spike", "huge_spike"):
        j = Lkv - 70
        gain = 6.0 if pattern == "late_spike" else 60.0
        for h in range(H):
            k[j, h * dh:(h + 1) * dh] = wl.round_to_bf16(gain * np.sign(q[nq // 2, h * dh:(h + 1) * dh]))
    scale = np.float32(np.log2(np.e) / np.sqrt(dh))
    qs = wl.round_to_bf16(q * scale)                          # what the kernel receives
    q_eff = qs.astype(np.float64) / float(scale)              # the queries the kernel then computes with
    K, Vt, Lp = _kv_buffers(k, v, H, dh, BF)
    got = _pkg().pf_op_attention(_dev(qs, BF), K, Vt, Lkv, Lp, H, dh, splits=splits, path=_pkg().PF_PATH_AUTO_PRESCALED_Q)
    torch.cuda.synchronize()
    name = _pkg().load_library().pf_attention_kernel_name(1, 0, dh, nq, 1).decode()
    assert name.split("<")[1].split(",")[2] == "true"
    assert torch.isfinite(got.float()).all()
    excess = _attention_error_over_bar(got, q_eff, k, v, H)
    _log("  max error / bar", excess)
    assert excess <= 1.0


@pytest.mark.parametrize("dh", [64, 72, 128])
@pytest.mark.parametrize("nq,Lkv,splits", [(1030, 50, 1), (1024, 128, 1), (1100, 190, 1), (1281, 256, 1), (1030, 300, 1),
                                           (1030, 448, 1), (1100, 1300, 3), (1025, 600, 5)])
def test_attention_prescaled_queries_short_key_ranges(dh, nq, Lkv, splits):
    """The 8-wave kernels with prescaled queries keep the first tile of a split, the steps up to the ring's first stage
    and the last up to three steps outside their tile loop: key ranges of one to seven tiles per split, every residue
    mod 4, ragged query and key tails, and splits that get no tile at all."""
    _log("attention prescaled short", dh, nq, Lkv, splits)
    H = 2
    rng = _rng(dh * 104729 + nq * 17 + Lkv)
    q, k, v = _draw(rng, (nq, H * dh), BF, 2.0), _draw(rng, (Lkv, H * dh), BF), _draw(rng, (Lkv, H * dh), BF)
    scale = np.float32(np.log2(np.e) / np.sqrt(dh))
    qs = wl.round_to_bf16(q * scale)
    q_eff = qs.astype(np.float64) / float(scale)
    K, Vt, Lp = _kv_buffers(k, v, H, dh, BF)
    got = _pkg().pf_op_attention(_dev(qs, BF), K, Vt, Lkv, Lp, H, dh, splits=splits, path=_pkg().PF_PATH_AUTO_PRESCALED_Q)
    torch.cuda.synchronize()
    assert _pkg().load_library().pf_attention_kernel_name(1, 0, dh, nq, 1).decode().split("<")[1].split(",")[3].rstrip(">") == "8"
    assert torch.isfinite(got.float()).all()
    excess = _attention_error_over_bar(got, q_eff, k, v, H)
    _log("  max error / bar", excess)
    assert excess <= 1.0


def test_attention_prescaled_path_rejects_other_kernels():
    pkg = _pkg()
    q = torch.zeros(8, 80, device="cuda", dtype=BF)
    K = torch.zeros(2, 128, 40, device="cuda", dtype=BF)
    Vt = torch.zeros(2, 40, 128, device="cuda", dtype=BF)
    with pytest.raises(pkg.PfError):
        pkg.pf_op_attention(q, K, Vt, 100, 128, 2, 40, path=pkg.PF_PATH_AUTO_PRESCALED_Q)      # head size without such a kernel
    with pytest.raises(pkg.PfError):
        pkg.pf_op_attention(q.float(), K.float(), Vt.float(), 100, 128, 2, 40, path=pkg.PF_PATH_AUTO_PRESCALED_Q)


def test_attention_ignores_finite_padding_rows():
    """Rows beyond kv_rows never contribute, whatever finite values they hold."""
    H, dh, nq, Lkv = 2, 72, 50, 300
    rng = _rng(123)
    q, k, v = _draw(rng, (nq, H * dh), BF), _draw(rng, (Lkv, H * dh), BF), _draw(rng, (Lkv, H * dh), BF)
    K, Vt, Lp = _kv_buffers(k, v, H, dh, BF)
    a = _pkg().pf_op_attention(_dev(q, BF), K, Vt, Lkv, Lp, H, dh)
    K[:, Lkv:] = 50.0
    Vt[:, :, Lkv:] = -1000.0
    b = _pkg().pf_op_attention(_dev(q, BF), K, Vt, Lkv, Lp, H, dh)
    torch.cuda.synchronize()
    assert torch.equal(a, b)


def test_op_argument_errors_do_not_launch():
    pkg = _pkg()
    x = torch.zeros(4, 12, device="cuda")
    with pytest.raises(pkg.PfError):
        pkg.pf_op_ln_modulate(x, x[0], x[0], 1e-6, F32)                  # d not a multiple of 8
    A = torch.zeros(8, 20, device="cuda")
    with pytest.raises(pkg.PfError):
        pkg.pf_op_gemm(A, A, None)                                       # K not a multiple of 8


def test_mfma_loop_probe_reports_a_plausible_rate():
    """The measurement aid behind bench.py's measured matrix ceiling: above the fp32 vector peak, below the sheet figure."""
    tf = _pkg().probe_mfma_tflops(workgroups=512, iters=500)
    _log("mfma loop", tf)
    assert 300.0 < tf < 2600.0
