"""Host-side checks of the C boundary that need no GPU: the library loads, exports every symbol the header
declares, validates configurations and call order before anything would be launched, and sizes the K/V
buffer as Sec. 3.4 (Table 1) says: full-sequence K and V for the stage's own layers."""
import ctypes as C
import os
import re

import pytest

import workloads as wl
from paper_2405_14430_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2405_14430_amd.build import build
        build()
    return B.load_library()


def test_header_symbols_are_exported(lib):
    text = open(os.path.join(ROOT, "include", "pfstage.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(pf_[a-z_0-9]+)\s*\(", text))
    assert {"pf_stage_create", "pf_kv_init", "pf_stage_patch_forward", "pf_kv_view"} <= declared
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(B.EXPORTS)


def test_kv_bytes_is_full_sequence_kv_for_own_layers(lib):
    for name, cfg in wl.CONFIGS.items():
        c = B.make_config(cfg)
        esz = 2 if cfg["dtype"] == "bf16" else 4
        Lp = (wl.kv_rows(cfg) + 127) // 128 * 128
        per_layer = 2 * Lp * cfg["hidden"] * esz
        if cfg["kind"] == 1:
            per_layer += 2 * ((cfg["text_len"] + 127) // 128 * 128) * cfg["hidden"] * esz
        assert lib.pf_stage_kv_bytes(C.byref(c)) == per_layer * cfg["n_layers"], name
        # halving the layers of the stage halves the buffer: the (1/N)(KV)L entry of Table 1
        if cfg["n_layers"] % 2 == 0:
            c2 = B.make_config(cfg, n_layers=cfg["n_layers"] // 2)
            assert lib.pf_stage_kv_bytes(C.byref(c2)) * 2 == lib.pf_stage_kv_bytes(C.byref(c))
        assert lib.pf_stage_workspace_bytes(C.byref(c)) > 0


def test_batch_multiplies_the_kv_buffer_and_limits(lib):
    """Every image of a batched call has K/V buffers of its own; batch 0 and 1 both mean one image."""
    for name in ("C2", "C3", "K3f"):
        cfg = wl.CONFIGS[name]
        one = lib.pf_stage_kv_bytes(C.byref(B.make_config(cfg)))
        assert lib.pf_stage_kv_bytes(C.byref(B.make_config(dict(cfg, batch=0)))) == one
        for b in (2, 3, 8):
            assert lib.pf_stage_kv_bytes(C.byref(B.make_config(dict(cfg, batch=b)))) == b * one
            assert lib.pf_stage_workspace_bytes(C.byref(B.make_config(dict(cfg, batch=b)))) > \
                lib.pf_stage_workspace_bytes(C.byref(B.make_config(cfg)))
        for b in (-1, 9):
            assert lib.pf_stage_kv_bytes(C.byref(B.make_config(dict(cfg, batch=b)))) == 0


def test_batched_views_and_plan(lib):
    cfg = dict(wl.CONFIGS["C2"], batch=2)
    st, h = _fake_stage(lib, cfg)
    assert st == 0
    v0, v1, vx = B.PfKvView(), B.PfKvView(), B.PfKvView()
    assert lib.pf_kv_view_image(h, 0, 0, 0, C.byref(v0)) == 0
    assert lib.pf_kv_view_image(h, 0, 1, 0, C.byref(v1)) == 0
    Lp = (wl.kv_rows(cfg) + 127) // 128 * 128
    assert v1.k - v0.k == Lp * cfg["hidden"] * 2 and v1.v - v0.v == Lp * cfg["hidden"] * 2
    assert v0.v - v0.k == 2 * Lp * cfg["hidden"] * 2          # both images' K come before the first V^T
    assert lib.pf_kv_view_image(h, 0, 2, 0, C.byref(vx)) == -6
    assert lib.pf_kv_view_image(h, 0, 1, 1, C.byref(vx)) == 0
    for nq in (wl.patch_rows(cfg), cfg["seq_img"]):
        sp, need, res = C.c_int(), C.c_size_t(), C.c_size_t()
        assert lib.pf_stage_attention_plan(h, nq, 0, C.byref(sp), C.byref(need), C.byref(res)) == 0
        assert need.value <= res.value
    lib.pf_stage_destroy(h)


BAD = [dict(qk_norm=2), dict(joint_rope=1), dict(txt_pre_only_last=1), dict(txt_pre_only_last=3), dict(qk_norm=1, head_dim=48, n_heads=8), dict(hidden=100), dict(n_patches=7), dict(head_dim=12, n_heads=32), dict(dtype_code=5), dict(kind=9),
       dict(grid_w=3), dict(mlp_dim=100), dict(n_layers=0), dict(ln_eps=0.0)]


@pytest.mark.parametrize("bad", BAD)
def test_invalid_configs_are_rejected(lib, bad):
    cfg = dict(wl.CONFIGS["C1"])
    code = bad.pop("dtype_code", None) if "dtype_code" in bad else None
    cfg.update(bad)
    c = B.make_config(cfg)
    if code is not None:
        c.dtype = code
    assert lib.pf_stage_kv_bytes(C.byref(c)) == 0
    kv = C.c_void_p(0x1000)
    out = C.c_void_p()
    layers = (B.PfLayerWeights * 1)()
    st = lib.pf_stage_create(C.byref(c), layers, kv, 1 << 40, kv, 1 << 40, None, C.byref(out))
    assert st in (-2, -4) and not out.value
    assert lib.pf_last_error(None)


def _fake_stage(lib, cfg):
    """A stage over fake (never dereferenced) device pointers: legal as long as nothing is launched."""
    c = B.make_config(cfg)
    layers = (B.PfLayerWeights * cfg["n_layers"])()
    txt = (B.PfLayerWeights * cfg["n_layers"])()
    for lw, tw in zip(layers, txt):
        for f in B._W_FIELDS:
            setattr(lw, f, 0x100000)
            setattr(tw, f, 0x100000)
        if cfg["kind"] == 2:
            lw.txt = C.pointer(tw)
    h = C.c_void_p()
    st = lib.pf_stage_create(C.byref(c), layers, C.c_void_p(0x200000), 1 << 40, C.c_void_p(0x300000), 1 << 40, None,
                             C.byref(h))
    return st, h


def test_create_argument_errors(lib):
    cfg = wl.CONFIGS["C1"]
    c = B.make_config(cfg)
    layers = (B.PfLayerWeights * 1)()
    h = C.c_void_p()
    assert lib.pf_stage_create(None, layers, C.c_void_p(256), 1, C.c_void_p(256), 1, None, C.byref(h)) == -1
    assert lib.pf_stage_create(C.byref(c), layers, C.c_void_p(0x200000), 16, C.c_void_p(0x300000), 1 << 40, None,
                               C.byref(h)) == -7                       # kv buffer too small
    assert lib.pf_stage_create(C.byref(c), layers, C.c_void_p(0x200008), 1 << 40, C.c_void_p(0x300000), 1 << 40, None,
                               C.byref(h)) == -7                       # misaligned
    assert lib.pf_stage_create(C.byref(c), layers, C.c_void_p(0x200000), 1 << 40, C.c_void_p(0x300000), 1 << 40, None,
                               C.byref(h)) == -1                       # null weight pointers
    assert b"null" in lib.pf_last_error(None)


def test_call_order_and_ranges_without_launching(lib):
    st, h = _fake_stage(lib, wl.CONFIGS["C1"])
    assert st == 0 and h.value
    cond = B.PfCond(cond=0x400000, text=None, text_out=None)
    x = C.c_void_p(0x500000)
    assert lib.pf_stage_patch_forward(h, x, C.byref(cond), 0, x) == -5            # before pf_kv_init
    assert b"pf_kv_init" in lib.pf_last_error(h)
    assert lib.pf_stage_patch_forward(h, None, C.byref(cond), 0, x) == -1
    assert lib.pf_stage_patch_forward(None, x, C.byref(cond), 0, x) == -1
    v = B.PfKvView()
    assert lib.pf_kv_view(h, 0, C.byref(v)) == 0
    assert v.rows == 256 and v.rows_padded == 256 and v.elem_bytes == 4 and v.v_row_stride == 1
    assert lib.pf_kv_view(h, 1, C.byref(v)) == -6
    assert lib.pf_xattn_kv_view(h, 0, C.byref(v)) == -2
    lib.pf_stage_destroy(h)
    lib.pf_stage_destroy(None)                                                     # NULL-safe
    # kind 1 needs the text features at pf_kv_init; checked before any launch
    st, h = _fake_stage(lib, wl.CONFIGS["C2s"])
    assert st == 0
    empty = B.PfCond(cond=None, text=None, text_out=None)
    assert lib.pf_kv_init(h, None, C.byref(empty), None) == -1
    lib.pf_stage_destroy(h)


def test_status_strings(lib):
    assert lib.pf_status_str(0) == b"PF_OK" and lib.pf_status_str(-5) == b"PF_ERR_STATE"


def test_op_argument_checks_without_launching(lib):
    p = C.c_void_p(0x100000)
    assert lib.pf_op_gemm(1, 0, p, 20, p, 20, None, p, 64, 4, 64, 20, 0, 64, 1, None, None, 0, None, 0, None) == -3
    assert lib.pf_op_gemm(7, 0, p, 24, p, 24, None, p, 64, 4, 64, 24, 0, 64, 1, None, None, 0, None, 0, None) == -4
    assert lib.pf_op_attention(1, 0, p, 64, p, p, 0, 128, 1, 64, p, 64, 4, 1, None, 0, None) == -3      # no key rows
    assert lib.pf_op_attention(1, 0, p, 64, p, p, 100, 128, 1, 64, p, 64, 4, 2, None, 0, None) == -7    # no workspace
    assert lib.pf_op_kv_scatter(1, p, 192, p, p, 128, 1, 64, 100, 64, 0, -1, 1, 1e4, None, None, 0.0, None) == -3   # rows overflow
    assert lib.pf_op_kv_scatter(1, p, 192, p, p, 128, 1, 64, 0, 64, 0, -1, 1, 1e4, p, None, 1e-6, None) == -1      # one norm weight only
    assert lib.pf_op_kv_scatter(1, p, 3 * 72, p, p, 128, 1, 72, 0, 64, 0, -1, 1, 1e4, p, p, 1e-6, None) == -3      # head_dim not a power of two
    assert lib.pf_op_ln_modulate(0, p, 12, p, p, 1e-6, p, 12, 4, 12, 1, None) == -3


def test_prescaled_query_path_is_checked_before_any_launch(lib):
    text = open(os.path.join(ROOT, "include", "pfstage.h")).read()
    for name in ("PF_PATH_AUTO", "PF_PATH_SIMT", "PF_PATH_AUTO_PRESCALED_Q"):
        assert int(re.search(name + r"\s*=\s*(\d+)", text).group(1)) == getattr(B, name)
    p = C.c_void_p(0x100000)
    q = B.PF_PATH_AUTO_PRESCALED_Q
    assert lib.pf_op_attention(0, q, p, 64, p, p, 100, 128, 1, 64, p, 64, 4, 1, None, 0, None) == -3      # fp32 has no such kernel
    assert lib.pf_op_attention(1, q, p, 40, p, p, 100, 128, 1, 40, p, 40, 4, 1, None, 0, None) == -3      # nor has head size 40
    assert b"PRESCALED" in lib.pf_last_error(None)
    assert lib.pf_op_attention_static(1, q, p, 96, p, p, 100, 128, 1, 96, p, 96, 4, 1, None) == -3


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5", "C3s", "C4s"])
def test_attention_partials_always_fit_the_reserved_workspace(lib, name):
    """Whatever row count a call has (image-only patch, patch plus joint text rows, warm-up pass, anything
    between), the split-KV partial results stay inside the workspace region reserved for them."""
    cfg = wl.CONFIGS[name]
    st, h = _fake_stage(lib, cfg)
    assert st == 0
    n, Lkv, Tj = wl.patch_rows(cfg), wl.kv_rows(cfg), wl.joint_text_rows(cfg)
    splits, need, have = C.c_int(), C.c_size_t(), C.c_size_t()
    probe = sorted({1, 63, 64, 65, 127, 128, 129, n - 1, n, n + 1, n + Tj, Lkv // 2, Lkv - 1, Lkv} & set(range(1, Lkv + 1)))
    for nq in probe + list(range(1, Lkv + 1, max(1, Lkv // 257))):
        for cross in ([0, 1] if cfg["kind"] == 1 else [0]):
            assert lib.pf_stage_attention_plan(h, nq, cross, C.byref(splits), C.byref(need), C.byref(have)) == 0
            assert need.value <= have.value and splits.value >= 1, (nq, cross)
    assert lib.pf_stage_attention_plan(h, Lkv + 1, 0, C.byref(splits), C.byref(need), C.byref(have)) == -6
    lib.pf_stage_destroy(h)


def test_stages_created_and_planned_on_two_threads_agree(lib):
    """No process-wide state takes part in a stage's launch plan: stages built and queried concurrently on two host
    threads (each stage used by its own thread only) report what a stage built alone reports."""
    import threading

    names = ["C2", "C3", "C4", "C5", "C2s", "C4s"]

    def plans(name):
        cfg = wl.CONFIGS[name]
        st, h = _fake_stage(lib, cfg)
        assert st == 0
        out = [lib.pf_stage_workspace_bytes(C.byref(B.make_config(cfg)))]
        splits, need, have = C.c_int(), C.c_size_t(), C.c_size_t()
        for nq in (1, wl.patch_rows(cfg), wl.kv_rows(cfg)):
            for cross in ([0, 1] if cfg["kind"] == 1 else [0]):
                assert lib.pf_stage_attention_plan(h, nq, cross, C.byref(splits), C.byref(need), C.byref(have)) == 0
                out.append((nq, cross, splits.value, need.value, have.value))
        n, d = wl.patch_rows(cfg), cfg["hidden"]
        out.append(lib.pf_gemm_kernel_name(1, 0, n, 3 * d, d))
        out.append(lib.pf_attention_kernel_name(1, 0, cfg["head_dim"], n, 1))
        lib.pf_stage_destroy(h)
        return out

    alone = {nm: plans(nm) for nm in names}
    got = [dict(), dict()]

    def worker(slot, order):
        for _ in range(20):
            for nm in order:
                got[slot][nm] = plans(nm)

    ts = [threading.Thread(target=worker, args=(0, names)), threading.Thread(target=worker, args=(1, names[::-1]))]
    for t in ts:
        t.start()
    for t in ts:
        t.join()
    assert got[0] == alone and got[1] == alone


def test_gemm_tile_entry_checks_without_launching(lib):
    p = C.c_void_p(0x100000)
    n = lib.pf_gemm_tile_count()
    assert n >= 1
    args = (1, 0, p, 64, p, 64, None, p, 64, 4, 64, 64, 0, 64, 1, None, None, 0, None, 0, None)
    assert lib.pf_op_gemm_tile(n + 1, *args) == -6 and lib.pf_op_gemm_tile(-1, *args) == -6
    assert lib.pf_op_gemm_tile(1, 0, *args[1:]) == -3            # tiles exist for bf16 only
    assert lib.pf_op_gemm_tile(1, 1, 0, p, 72, p, 72, None, p, 64, 4, 64, 72, 0, 64, 1, None, None, 0, None, 0, None) == -3


def test_static_scratch_entry_rejects_oversize_before_touching_the_device(lib):
    """The entry point that allocates nothing has a fixed array for its split partials: a launch that needs more is
    refused on the host, before any device call, with a message that names the sizes."""
    p = C.c_void_p(0x100000)
    cap = lib.pf_static_scratch_bytes()
    assert cap == 32 << 20
    assert lib.pf_op_attention_ws_bytes(4096, 16, 72, 8) > cap
    assert lib.pf_op_attention_static(1, 0, p, 1152, p, p, 4096, 4096, 16, 72, p, 1152, 4096, 8, None) == -7
    msg = lib.pf_last_error(None)
    assert b"static scratch" in msg and str(cap).encode() in msg
    assert lib.pf_op_attention_static(1, 0, p, 1152, p, p, 0, 4096, 16, 72, p, 1152, 64, 2, None) == -3     # no key rows
    assert lib.pf_op_attention_static(1, 0, None, 1152, p, p, 128, 128, 16, 72, p, 1152, 64, 2, None) == -1


def _tile_map(lib, M, N, bm, bn):
    grid, tm, tn = C.c_uint(0), C.c_int(0), C.c_int(0)
    assert lib.pf_gemm_tile_map(M, N, bm, bn, 0, C.byref(grid), C.byref(tm), C.byref(tn)) in (0, 1)
    tiles = {}
    for wg in range(grid.value):
        r = lib.pf_gemm_tile_map(M, N, bm, bn, wg, C.byref(grid), C.byref(tm), C.byref(tn))
        assert r in (0, 1)
        if r:
            tiles.setdefault((tm.value, tn.value), []).append(wg)
    return grid.value, tiles


@pytest.mark.parametrize("M,N,bm,bn", [
    (2048, 9216, 128, 192), (2048, 12288, 256, 192), (2048, 3072, 128, 192),      # Flux-scale projections
    (4096, 3456, 128, 128), (4096, 1152, 128, 128), (512, 3456, 64, 64), (512, 1152, 64, 64),
    (666, 4608, 64, 64), (77, 1000, 64, 64), (1, 8, 64, 64), (130, 70, 128, 64), (5000, 40, 256, 256),
    (64, 100000, 64, 64), (100000, 64, 128, 128)])
def test_gemm_workgroup_to_tile_map_covers_every_tile_once_and_keeps_an_xcd_in_one_block(lib, M, N, bm, bn):
    """Host view of the GEMM kernels' workgroup -> tile map: every output tile has exactly one workgroup, the padded
    grid stays within 9/8 of the tile count plus one row of eight, and the workgroups of one XCD (ids congruent mod 8)
    cover one rectangle of the tile grid - the point of the map: an XCD's L2 then holds one block's operand panels."""
    tiles_m, tiles_n = -(-M // bm), -(-N // bn)
    grid, tiles = _tile_map(lib, M, N, bm, bn)
    assert sorted(tiles) == [(i, j) for i in range(tiles_m) for j in range(tiles_n)]
    assert all(len(v) == 1 for v in tiles.values())
    assert grid % 8 == 0 and grid >= tiles_m * tiles_n
    for x in range(8):
        mine = [t for t, wgs in tiles.items() if wgs[0] % 8 == x]
        if not mine:
            continue
        r0, r1 = min(t[0] for t in mine), max(t[0] for t in mine)
        c0, c1 = min(t[1] for t in mine), max(t[1] for t in mine)
        assert len(mine) == (r1 - r0 + 1) * (c1 - c0 + 1)          # a full rectangle
    # past the grid and bad arguments
    g, a, b = C.c_uint(0), C.c_int(0), C.c_int(0)
    assert lib.pf_gemm_tile_map(M, N, bm, bn, grid, C.byref(g), C.byref(a), C.byref(b)) == 0 and a.value == -1
    assert lib.pf_gemm_tile_map(M, N, bm, bn, 0, None, C.byref(a), C.byref(b)) == -1
    assert lib.pf_gemm_tile_map(0, N, bm, bn, 0, C.byref(g), C.byref(a), C.byref(b)) == -6


def test_gemm_tile_map_cuts_the_flux_mlp_down_grid_two_by_four(lib):
    """2048 x 3072 with 128 x 192 tiles (16 x 16 tiles): the cut with the fewest operand rows per XCD is 2 along M and
    4 along N (8 x 128 + 4 x 192 = 1792 rows against 2048 for 4 x 2 and 2432 for 1 x 8), without padding."""
    grid, tiles = _tile_map(lib, 2048, 3072, 128, 192)
    assert grid == 256
    mine = sorted(t for t, wgs in tiles.items() if wgs[0] % 8 == 0)
    assert mine[0] == (0, 0) and mine[-1] == (7, 3) and len(mine) == 32


def test_build_refuses_an_attention_kernel_that_spills():
    """The attention kernels' LDS fragment reads are asynchronous loads tracked by hand, so a register spill makes them
    wrong, not slow: the build reads the compiler's per-kernel resource remarks and refuses scratch use."""
    from paper_2405_14430_amd import build as bld
    def log(scratch, spill):
        return ("a.hip:1:1: remark: Function Name: _ZN2pf17attn_mfma2_kernelILi128EEEv [-Rpass-analysis=kernel-resource-usage]\n"
                f"a.hip:1:1: remark:     ScratchSize [bytes/lane]: {scratch} [-Rpass-analysis=kernel-resource-usage]\n"
                f"a.hip:1:1: remark:     VGPRs Spill: {spill} [-Rpass-analysis=kernel-resource-usage]\n")
    bld._check_no_scratch("attn_mfma2.hip", log(0, 0))
    bld._check_no_scratch("gemm_mfma_dl.hip", log(64, 3))          # not a checked source
    for bad in (log(24, 0), log(0, 2), "no remarks at all"):
        with pytest.raises(RuntimeError):
            bld._check_no_scratch("attn_mfma2.hip", bad)
