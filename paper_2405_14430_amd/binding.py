"""ctypes binding of libpfstage.so: argument marshalling only.

Function names mirror include/pfstage.h.  torch is used for device memory and streams;
every arithmetic step runs inside the library's HIP kernels.  Loading fails loudly when the
library has not been built (python paper_2405_14430_amd/build.py, or __graft_entry__.build()).
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpfstage.so")

PF_F32, PF_BF16 = 0, 1
PF_PATH_AUTO, PF_PATH_SIMT, PF_PATH_AUTO_PRESCALED_Q = 0, 1, 2
KERNEL_CLASSES = ["modulation", "ln_modulate", "gemm_qkv", "kv_scatter", "attention", "attn_combine",
                  "gemm_out", "gemm_xattn", "xattn", "gemm_up", "gemm_down", "copy"]
STATUS = {0: "PF_OK", -1: "PF_ERR_NULL", -2: "PF_ERR_CONFIG", -3: "PF_ERR_SHAPE", -4: "PF_ERR_DTYPE",
          -5: "PF_ERR_STATE", -6: "PF_ERR_RANGE", -7: "PF_ERR_WORKSPACE", -8: "PF_ERR_DEVICE"}


class PfConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("kind", "dtype", "n_layers", "hidden", "n_heads", "head_dim", "mlp_dim",
                                          "seq_img", "n_patches", "text_len", "cross_dim", "grid_h", "grid_w")] + \
               [("ln_eps", C.c_float), ("rope_theta", C.c_float), ("gelu_tanh", C.c_int32), ("kernel_path", C.c_int32), ("batch", C.c_int32),
                ("qk_norm", C.c_int32), ("joint_rope", C.c_int32), ("txt_pre_only_last", C.c_int32)]


class PfLayerWeights(C.Structure):
    pass


_W_FIELDS = ["w_mod", "b_mod", "w_qkv", "b_qkv", "w_o", "b_o", "w_up", "b_up", "w_down", "b_down",
             "xattn_wq", "xattn_bq", "xattn_wkv", "xattn_bkv", "xattn_wo", "xattn_bo", "q_norm_w", "k_norm_w"]
PfLayerWeights._fields_ = [(n, C.c_void_p) for n in _W_FIELDS] + [("txt", C.POINTER(PfLayerWeights))]


class PfCond(C.Structure):
    _fields_ = [("cond", C.c_void_p), ("text", C.c_void_p), ("text_out", C.c_void_p), ("same_cond", C.c_int32)]


class PfKvView(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p), ("rows", C.c_int32), ("rows_padded", C.c_int32),
                ("text_rows", C.c_int32), ("elem_bytes", C.c_int32),
                ("k_row_stride", C.c_int64), ("k_head_stride", C.c_int64), ("k_col_stride", C.c_int64),
                ("v_row_stride", C.c_int64), ("v_head_stride", C.c_int64), ("v_col_stride", C.c_int64)]


EXPORTS = ["pf_stage_kv_bytes", "pf_stage_workspace_bytes", "pf_stage_create", "pf_kv_init",
           "pf_stage_patch_forward", "pf_kv_view", "pf_xattn_kv_view", "pf_stage_attention_plan", "pf_stage_set_stream",
           "pf_stage_profile",
           "pf_stage_profile_read", "pf_stage_destroy", "pf_status_str", "pf_last_error", "pf_op_modulation",
           "pf_op_ln_modulate", "pf_op_gemm", "pf_op_kv_scatter", "pf_op_attention_ws_bytes", "pf_op_attention", "pf_attention_kernel_name", "pf_probe_mfma_loop",
           "pf_gemm_tile_count", "pf_gemm_tile_map", "pf_op_gemm_tile", "pf_static_scratch_bytes", "pf_op_attention_static", "pf_gemm_kernel_name", "pf_op_axpy", "pf_kv_view_image", "pf_op_axpby"]

_lib = None


def load_library():
    """dlopen libpfstage.so and declare the prototypes.  Raises if the library is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it first (python paper_2405_14430_amd/build.py). "
                           "There is no fallback path.")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64, f32, sz = C.c_void_p, C.c_int, C.c_int64, C.c_float, C.c_size_t
    lib.pf_stage_kv_bytes.restype = sz
    lib.pf_stage_kv_bytes.argtypes = [C.POINTER(PfConfig)]
    lib.pf_stage_workspace_bytes.restype = sz
    lib.pf_stage_workspace_bytes.argtypes = [C.POINTER(PfConfig)]
    lib.pf_stage_create.restype = i32
    lib.pf_stage_create.argtypes = [C.POINTER(PfConfig), C.POINTER(PfLayerWeights), vp, sz, vp, sz, vp, C.POINTER(vp)]
    lib.pf_kv_init.restype = i32
    lib.pf_kv_init.argtypes = [vp, vp, C.POINTER(PfCond), vp]
    lib.pf_stage_patch_forward.restype = i32
    lib.pf_stage_patch_forward.argtypes = [vp, vp, C.POINTER(PfCond), i32, vp]
    lib.pf_kv_view.restype = i32
    lib.pf_kv_view.argtypes = [vp, i32, C.POINTER(PfKvView)]
    lib.pf_xattn_kv_view.restype = i32
    lib.pf_xattn_kv_view.argtypes = [vp, i32, C.POINTER(PfKvView)]
    lib.pf_kv_view_image.restype = i32
    lib.pf_kv_view_image.argtypes = [vp, i32, i32, i32, C.POINTER(PfKvView)]
    lib.pf_stage_attention_plan.restype = i32
    lib.pf_stage_attention_plan.argtypes = [vp, i32, i32, C.POINTER(C.c_int), C.POINTER(sz), C.POINTER(sz)]
    lib.pf_stage_set_stream.restype = i32
    lib.pf_stage_set_stream.argtypes = [vp, vp]
    lib.pf_stage_profile.restype = i32
    lib.pf_stage_profile.argtypes = [vp, i32]
    lib.pf_stage_profile_read.restype = i32
    lib.pf_stage_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    lib.pf_stage_destroy.restype = None
    lib.pf_stage_destroy.argtypes = [vp]
    lib.pf_status_str.restype = C.c_char_p
    lib.pf_status_str.argtypes = [i32]
    lib.pf_last_error.restype = C.c_char_p
    lib.pf_last_error.argtypes = [vp]
    lib.pf_op_modulation.restype = i32
    lib.pf_op_modulation.argtypes = [i32, vp, vp, vp, vp, i32, i32, i32, vp]
    lib.pf_op_ln_modulate.restype = i32
    lib.pf_op_ln_modulate.argtypes = [i32, vp, i64, vp, vp, f32, vp, i64, i32, i32, i32, vp]
    lib.pf_op_gemm.restype = i32
    lib.pf_op_gemm.argtypes = [i32, i32, vp, i64, vp, i64, vp, vp, i64, i32, i32, i32, i32, i32, i32, vp, vp, i64,
                               vp, i64, vp]
    lib.pf_op_kv_scatter.restype = i32
    lib.pf_op_kv_scatter.argtypes = [i32, vp, i64, vp, vp, i32, i32, i32, i32, i32, i32, i32, i32, f32, vp, vp, f32, vp]
    lib.pf_attention_kernel_name.restype = C.c_char_p
    lib.pf_attention_kernel_name.argtypes = [i32, i32, i32, i32, i32]
    lib.pf_probe_mfma_loop.restype = i32
    lib.pf_probe_mfma_loop.argtypes = [vp, i32, i32, C.POINTER(C.c_double), vp]
    lib.pf_op_attention_ws_bytes.restype = sz
    lib.pf_op_attention_ws_bytes.argtypes = [i32, i32, i32, i32]
    lib.pf_op_attention.restype = i32
    lib.pf_op_attention.argtypes = [i32, i32, vp, i64, vp, vp, i32, i32, i32, i32, vp, i64, i32, i32, vp, sz, vp]
    lib.pf_static_scratch_bytes.restype = sz
    lib.pf_static_scratch_bytes.argtypes = []
    lib.pf_op_attention_static.restype = i32
    lib.pf_op_attention_static.argtypes = [i32, i32, vp, i64, vp, vp, i32, i32, i32, i32, vp, i64, i32, i32, vp]
    lib.pf_gemm_kernel_name.restype = C.c_char_p
    lib.pf_gemm_kernel_name.argtypes = [i32, i32, i32, i32, i32]
    lib.pf_op_axpy.restype = i32
    lib.pf_op_axpy.argtypes = [vp, vp, f32, vp, i64, vp]
    lib.pf_op_axpby.restype = i32
    lib.pf_op_axpby.argtypes = [vp, vp, f32, f32, vp, i64, vp]
    lib.pf_gemm_tile_count.restype = i32
    lib.pf_gemm_tile_count.argtypes = []
    lib.pf_gemm_tile_map.restype = i32
    lib.pf_gemm_tile_map.argtypes = [i32, i32, i32, i32, C.c_uint, C.POINTER(C.c_uint), C.POINTER(i32), C.POINTER(i32)]
    lib.pf_op_gemm_tile.restype = i32
    lib.pf_op_gemm_tile.argtypes = [i32] + lib.pf_op_gemm.argtypes
    _lib = lib
    return lib


class PfError(RuntimeError):
    def __init__(self, status, msg=""):
        self.status = status
        super().__init__(f"{STATUS.get(status, status)}: {msg}")


def make_config(cfg, kernel_path=PF_PATH_AUTO, n_layers=None):
    return PfConfig(kind=cfg["kind"], dtype=PF_BF16 if cfg["dtype"] == "bf16" else PF_F32,
                    n_layers=cfg["n_layers"] if n_layers is None else n_layers, hidden=cfg["hidden"],
                    n_heads=cfg["n_heads"], head_dim=cfg["head_dim"], mlp_dim=cfg["mlp_dim"],
                    seq_img=cfg["seq_img"], n_patches=cfg["n_patches"], text_len=cfg.get("text_len", 0),
                    cross_dim=cfg.get("cross_dim", 0), grid_h=cfg["grid_h"], grid_w=cfg["grid_w"],
                    ln_eps=cfg.get("ln_eps", 1e-6), rope_theta=cfg.get("rope_theta", 1e4),
                    gelu_tanh=cfg.get("gelu_tanh", 1), kernel_path=kernel_path, batch=cfg.get("batch", 1),
                    qk_norm=cfg.get("qk_norm", 0), joint_rope=cfg.get("joint_rope", 0),
                    txt_pre_only_last=cfg.get("txt_pre_only_last", 0))


def torch_dtype(cfg):
    return torch.bfloat16 if cfg["dtype"] == "bf16" else torch.float32


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream_ptr(stream=None):
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def to_device(a, dtype, device="cuda"):
    """numpy float32 array (values already representable in dtype) -> device tensor of dtype."""
    return torch.from_numpy(np.ascontiguousarray(a)).to(device=device, dtype=dtype)


class Stage:
    """Owns the device memory of one stage (weights, K/V buffer, workspace) and forwards calls to the library."""

    def __init__(self, cfg, layers, kernel_path=PF_PATH_AUTO, device="cuda", stream=None):
        self.lib = load_library()
        self.cfg = dict(cfg)
        self.device = device
        self.dt = torch_dtype(cfg)
        self.c = make_config(cfg, kernel_path, n_layers=len(layers))
        self.n = cfg["seq_img"] // cfg["n_patches"]
        self.d = cfg["hidden"]
        self.T = cfg.get("text_len", 0)
        self.joint = cfg["kind"] in (2, 3)
        self._keep = []
        arr = (PfLayerWeights * len(layers))()
        self._txt = (PfLayerWeights * len(layers))()
        for i, w in enumerate(layers):
            self._fill(arr[i], w)
            if "txt" in w:
                self._fill(self._txt[i], w["txt"])
                arr[i].txt = C.pointer(self._txt[i])
        self._layers = arr
        kvb = self.lib.pf_stage_kv_bytes(C.byref(self.c))
        wsb = self.lib.pf_stage_workspace_bytes(C.byref(self.c))
        if kvb == 0:
            raise PfError(-2, "invalid configuration")
        self.kv = torch.zeros(kvb, dtype=torch.uint8, device=device)
        self.ws = torch.empty(wsb, dtype=torch.uint8, device=device)
        self.h = C.c_void_p()
        st = self.lib.pf_stage_create(C.byref(self.c), arr, _ptr(self.kv), kvb, _ptr(self.ws), wsb,
                                      _stream_ptr(stream), C.byref(self.h))
        if st != 0:
            raise PfError(st, self.lib.pf_last_error(None).decode())

    def _fill(self, dst, w):
        for name in _W_FIELDS:
            if name in w:
                t = to_device(w[name], self.dt, self.device)
                self._keep.append(t)
                setattr(dst, name, t.data_ptr())

    def _check(self, st):
        if st != 0:
            raise PfError(st, self.lib.pf_last_error(self.h).decode())

    def _cond(self, cond, text, text_out, same_cond=False):
        return PfCond(cond=None if cond is None else cond.data_ptr(), text=None if text is None else text.data_ptr(),
                      text_out=None if text_out is None else text_out.data_ptr(), same_cond=int(bool(same_cond)))

    def kv_init(self, x_prev=None, cond=None, text=None, want_output=False):
        """x_prev/cond/text: device tensors (x_prev, cond, joint text: float32; kind-1 text: stage dtype).  A stage with
        batch B > 1 takes every array with a leading image axis of length B."""
        y = torch.empty_like(x_prev) if (want_output and x_prev is not None) else None
        tout = torch.empty_like(text) if (want_output and self.joint and text is not None and x_prev is not None) else None
        pc = self._cond(cond, text, tout)
        self._check(self.lib.pf_kv_init(self.h, _ptr(x_prev), C.byref(pc), _ptr(y)))
        return (y, tout) if want_output else None

    def patch_forward(self, x_patch, cond, p, text=None, out=None, text_out=None, same_cond=False):
        """same_cond: `cond` has the values of this stage's previous call (the other patches of the same diffusion
        step): the stage reuses its modulation vectors instead of deriving them again."""
        y = torch.empty_like(x_patch) if out is None else out
        if self.joint and text is not None and text_out is None:
            text_out = torch.empty_like(text)
        pc = self._cond(cond, text if self.joint else None, text_out, same_cond)
        self._check(self.lib.pf_stage_patch_forward(self.h, _ptr(x_patch), C.byref(pc), int(p), _ptr(y)))
        return (y, text_out) if (self.joint and text is not None) else y

    def _view(self, layer, image, cross):
        v = PfKvView()
        self._check(self.lib.pf_kv_view_image(self.h, layer, image, int(cross), C.byref(v)))
        typed = self.kv.view(self.dt)
        H, dh, esz = self.cfg["n_heads"], self.cfg["head_dim"], v.elem_bytes
        ko = (v.k - self.kv.data_ptr()) // esz
        vo = (v.v - self.kv.data_ptr()) // esz
        K = typed.as_strided((v.rows, H, dh), (v.k_row_stride, v.k_head_stride, v.k_col_stride), ko)
        V = typed.as_strided((v.rows, H, dh), (v.v_row_stride, v.v_head_stride, v.v_col_stride), vo)
        return K, V, v

    def kv_view(self, layer, image=0):
        """(K, V) as strided [rows, H, dh] tensor views into the caller-owned buffer, plus the raw view struct."""
        return self._view(layer, image, False)

    def xattn_kv_view(self, layer, image=0):
        return self._view(layer, image, True)

    def set_stream(self, stream):
        self._check(self.lib.pf_stage_set_stream(self.h, _stream_ptr(stream)))

    def profile(self, enable):
        self._check(self.lib.pf_stage_profile(self.h, int(enable)))

    def profile_read(self):
        ms = (C.c_double * len(KERNEL_CLASSES))()
        cnt = (C.c_int64 * len(KERNEL_CLASSES))()
        self._check(self.lib.pf_stage_profile_read(self.h, ms, cnt))
        return {k: (ms[i], cnt[i]) for i, k in enumerate(KERNEL_CLASSES)}

    def destroy(self):
        if self.h:
            self.lib.pf_stage_destroy(self.h)
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


# ---- single-operator wrappers (device tensors in, device tensors out) ---------------------------------------
def _dt_code(t):
    return PF_BF16 if t.dtype == torch.bfloat16 else PF_F32


def _ok(st):
    if st != 0:
        raise PfError(st)


def pf_op_modulation(w, b, c, table_mode=False):
    lib = load_library()
    out_dim = w.numel() if table_mode else w.shape[0]
    in_dim = w.shape[-1]
    mod = torch.empty(out_dim, dtype=torch.float32, device=w.device)
    _ok(lib.pf_op_modulation(_dt_code(w), _ptr(w), _ptr(b), _ptr(c), _ptr(mod), out_dim, in_dim, int(table_mode),
                             _stream_ptr()))
    return mod


def pf_op_ln_modulate(x, shift, scale, eps, dtype, normalize=True):
    lib = load_library()
    rows, d = x.shape
    out = torch.empty(rows, d, dtype=dtype, device=x.device)
    _ok(lib.pf_op_ln_modulate(PF_BF16 if dtype == torch.bfloat16 else PF_F32, _ptr(x), x.stride(0), _ptr(shift),
                              _ptr(scale), eps, _ptr(out), out.stride(0), rows, d, int(normalize), _stream_ptr()))
    return out


def pf_op_gemm(A, W, bias, epilogue=0, gelu_from=None, gelu_tanh=1, gate=None, R=None, want_copy=False,
               path=PF_PATH_AUTO, tile=0):
    """epilogue 0 -> dtype [M,N]; epilogue 1 -> (float32 [M,N] new residual, optional dtype copy).
    tile > 0 goes through pf_op_gemm_tile (one tile configuration of the bf16 kernel, this launch only)."""
    lib = load_library()
    M, K = A.shape
    N = W.shape[0]
    if epilogue == 0:
        Cc = torch.empty(M, N, dtype=A.dtype, device=A.device)
        C2 = None
    else:
        Cc = torch.empty(M, N, dtype=torch.float32, device=A.device)
        C2 = torch.empty(M, N, dtype=A.dtype, device=A.device) if want_copy else None
    args = (_dt_code(A), path, _ptr(A), A.stride(0), _ptr(W), W.stride(0), _ptr(bias), _ptr(Cc),
            Cc.stride(0), M, N, K, epilogue, N if gelu_from is None else gelu_from, gelu_tanh, _ptr(gate),
            _ptr(R), 0 if R is None else R.stride(0), _ptr(C2), 0 if C2 is None else C2.stride(0), _stream_ptr())
    _ok(lib.pf_op_gemm_tile(int(tile), *args) if tile else lib.pf_op_gemm(*args))
    return Cc if epilogue == 0 else (Cc, C2)


def pf_op_kv_scatter(qkv, kbuf, vtbuf, rows_padded, n_heads, head_dim, row0, rope=False, tok0=-1, grid_w=1,
                     theta=1e4, q_norm_w=None, k_norm_w=None, norm_eps=1e-6):
    lib = load_library()
    _ok(lib.pf_op_kv_scatter(_dt_code(qkv), _ptr(qkv), qkv.stride(0), _ptr(kbuf), _ptr(vtbuf), rows_padded, n_heads,
                             head_dim, row0, qkv.shape[0], int(rope), tok0, grid_w, theta, _ptr(q_norm_w),
                             _ptr(k_norm_w), norm_eps, _stream_ptr()))


def pf_op_attention(q, kbuf, vtbuf, kv_rows, rows_padded, n_heads, head_dim, splits=1, path=PF_PATH_AUTO):
    lib = load_library()
    nq = q.shape[0]
    out = torch.empty(nq, n_heads * head_dim, dtype=q.dtype, device=q.device)
    wsb = lib.pf_op_attention_ws_bytes(nq, n_heads, head_dim, splits)
    ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device=q.device)
    _ok(lib.pf_op_attention(_dt_code(q), path, _ptr(q), q.stride(0), _ptr(kbuf), _ptr(vtbuf), kv_rows, rows_padded,
                            n_heads, head_dim, _ptr(out), out.stride(0), nq, splits, _ptr(ws), wsb, _stream_ptr()))
    return out


def pf_op_attention_static(q, kbuf, vtbuf, kv_rows, rows_padded, n_heads, head_dim, out, splits=1, path=PF_PATH_AUTO):
    """pf_op_attention through the entry point that allocates nothing: `out` is the caller's, the split partials go into
    the library's static scratch array."""
    lib = load_library()
    st = lib.pf_op_attention_static(_dt_code(q), path, _ptr(q), q.stride(0), _ptr(kbuf), _ptr(vtbuf), kv_rows, rows_padded,
                                    n_heads, head_dim, _ptr(out), out.stride(0), q.shape[0], splits, _stream_ptr())
    if st != 0:
        raise PfError(st, lib.pf_last_error(None).decode())
    return out


def probe_mfma_tflops(workgroups=512, iters=4000):
    """TFLOP/s of a register-only bf16 MFMA loop on the current device and stream (measured ceiling of the matrix pipes)."""
    lib = load_library()
    out = torch.empty(workgroups * 256, dtype=torch.float32, device="cuda")
    fl = C.c_double()
    _ok(lib.pf_probe_mfma_loop(_ptr(out), workgroups, 50, C.byref(fl), _stream_ptr()))      # warm-up
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    _ok(lib.pf_probe_mfma_loop(_ptr(out), workgroups, iters, C.byref(fl), _stream_ptr()))
    e1.record()
    e1.synchronize()
    return fl.value / (e0.elapsed_time(e1) * 1e-3) / 1e12


def pf_op_axpy(x, y, alpha, out=None):
    lib = load_library()
    out = torch.empty_like(x) if out is None else out
    _ok(lib.pf_op_axpy(_ptr(x), _ptr(y), float(alpha), _ptr(out), x.numel(), _stream_ptr()))
    return out


def pf_op_axpby(x, y, a, b, out=None):
    lib = load_library()
    out = torch.empty_like(x) if out is None else out
    _ok(lib.pf_op_axpby(_ptr(x), _ptr(y), float(a), float(b), _ptr(out), x.numel(), _stream_ptr()))
    return out
