"""CPU oracle for one PipeFusion pipeline stage working on one patch.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the HIP
library is checked against.  Only tests, the smoke check and the benchmark's
`cpu_baseline` leg may import it; the product path never does.  It shares no
code with the HIP path and imports nothing from it.

Everything is numpy in float64, with no intermediate rounding, no tiling, no
fusion and no reordering: each function is the textbook formula or the
paper's step written out.

What the paper fixes (PipeFusion, Sec. 3.3):
  * the input sequence is cut into M non-overlapping patches and the model into
    stages of consecutive layers;
  * a stage keeps, for every one of its layers, K and V of the FULL sequence
    (Sec. 3.4, Table 1: memory (1/N)(KV)L per device);
  * when the stage works on patch p at diffusion step T, the K/V rows of patch
    p are fresh (written before attending), rows written earlier in this step
    are fresh too, and every other row still holds what the previous step
    (T+1) left there;
  * warm-up steps run synchronously on the whole sequence with no stale
    activations (Sec. 3.3), and the buffer may also simply start at zero
    (App. B, ablation study).
What the paper only names (Sec. 2: "Multi-Head Self-Attention, Layer Norm and
Feedforward Networks") is filled in with the standard definitions of adaLN DiT
blocks; every such reading is listed in the design notes of this repository.

Parity pins (tests/test_oracle_pins.py): M = 1 and fresh-everywhere equal a
full-sequence forward written independently with torch.nn.functional; brute
force scalar loops on tiny shapes; the zero-buffer closed form; softmax row
sums; LayerNorm / GELU / RoPE identities; gate = 0 identity; permutation
invariance of the K/V rows.  The paper prints no numeric value for this path.
"""
from __future__ import annotations

import math

import numpy as np

KIND_ADALN_ZERO = 0
KIND_ADALN_SINGLE_XATTN = 1
KIND_MMDIT_JOINT = 2
KIND_SINGLE_STREAM = 3

F64 = np.float64


# --------------------------------------------------------------------------- #
# elementary operators                                                         #
# --------------------------------------------------------------------------- #
def silu(x):
    """x * sigmoid(x)."""
    x = np.asarray(x, F64)
    return x / (1.0 + np.exp(-x))


def gelu(x, tanh_approx=True):
    """GELU.  tanh form: 0.5 x (1 + tanh( sqrt(2/pi) (x + 0.044715 x^3) )); else the erf form."""
    x = np.asarray(x, F64)
    if tanh_approx:
        return 0.5 * x * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (x + 0.044715 * x ** 3)))
    erf = np.vectorize(math.erf, otypes=[F64])
    return 0.5 * x * (1.0 + erf(x / math.sqrt(2.0)))


def layer_norm(x, eps):
    """Per-row LayerNorm over the last axis, biased variance, no learned affine."""
    x = np.asarray(x, F64)
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps)


def ln_modulate(x, shift, scale, eps):
    """adaLN: LN(x) * (1 + scale) + shift, shift/scale broadcast over rows."""
    return layer_norm(x, eps) * (1.0 + np.asarray(scale, F64)) + np.asarray(shift, F64)


def linear(x, w, b):
    """y = x W^T + b with W stored [out_features, in_features]."""
    return np.asarray(x, F64) @ np.asarray(w, F64).T + np.asarray(b, F64)


def softmax_rows(s):
    s = np.asarray(s, F64)
    e = np.exp(s - s.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


def attention(q, k, v, n_heads, return_probs=False, weight_round=None):
    """Multi-head attention of queries q [nq, d] over keys/values k, v [nk, d].

    Head h owns columns [h*dh, (h+1)*dh).  Scores are scaled by 1/sqrt(dh).
    weight_round: None (exact), or the storage-rounding probe of StageOracle applied to the softmax weights
    before they multiply v.
    """
    q, k, v = (np.asarray(t, F64) for t in (q, k, v))
    nq, d = q.shape
    dh = d // n_heads
    out = np.empty((nq, d), F64)
    probs = []
    for h in range(n_heads):
        sl = slice(h * dh, (h + 1) * dh)
        p = softmax_rows((q[:, sl] @ k[:, sl].T) / math.sqrt(dh))
        if weight_round is not None:
            p = weight_round(p)
        out[:, sl] = p @ v[:, sl]
        if return_probs:
            probs.append(p)
    return (out, probs) if return_probs else out


def rms_norm_heads(t, w, n_heads, eps):
    """RMSNorm over the channels of each head: t [n, H*dh] -> t / sqrt(mean_c t^2 + eps) * w, w [dh] shared by heads."""
    t = np.asarray(t, F64)
    n, d = t.shape
    th = t.reshape(n, n_heads, d // n_heads)
    r = np.sqrt(np.mean(th * th, axis=-1, keepdims=True) + eps)
    return (th / r * np.asarray(w, F64)).reshape(n, d)


def rope_angles(rows, cols, head_dim, theta):
    """Rotation angles [n, head_dim/2] for tokens at grid positions (rows[i], cols[i]).

    The first half of the head's channels encodes the grid row, the second half
    the grid column.  Within an axis of width w = head_dim/2, channel pair
    (2i, 2i+1) turns by pos * theta^(-2i/w).
    """
    w = head_dim // 2
    freqs = theta ** (-(2.0 * np.arange(w // 2, dtype=F64)) / w)          # [w/2]
    ang_r = np.asarray(rows, F64)[:, None] * freqs[None, :]
    ang_c = np.asarray(cols, F64)[:, None] * freqs[None, :]
    return np.concatenate([ang_r, ang_c], axis=1)                          # [n, head_dim/2]


def rope_apply(t, angles, n_heads):
    """Rotate channel pairs (2j, 2j+1) of every head of t [n, d] by angles[:, j]."""
    t = np.asarray(t, F64)
    n, d = t.shape
    dh = d // n_heads
    th = t.reshape(n, n_heads, dh // 2, 2)
    c = np.cos(angles)[:, None, :]
    s = np.sin(angles)[:, None, :]
    out = np.empty_like(th)
    out[..., 0] = th[..., 0] * c - th[..., 1] * s
    out[..., 1] = th[..., 0] * s + th[..., 1] * c
    return out.reshape(n, d)


# --------------------------------------------------------------------------- #
# the stage                                                                    #
# --------------------------------------------------------------------------- #
class StageOracle:
    """A contiguous stack of DiT blocks with per-layer full-sequence K/V buffers.

    cfg: dict with kind, n_layers, hidden, n_heads, head_dim, mlp_dim, seq_img,
         n_patches, text_len, cross_dim, grid_h, grid_w, ln_eps, rope_theta,
         gelu_tanh; optional qk_norm (RMSNorm of q and k per head, before RoPE,
         eps = ln_eps, weights q_norm_w / k_norm_w [dh]) and joint_rope (kind 2:
         RoPE on the image rows as in kind 3) and txt_pre_only_last (kind 2: in
         the stack's last block the text stream only supplies keys and values -
         the final joint block of an MMDiT, whose text output nobody reads: its
         modulation has two chunks [shift, scale], its rows are normalised,
         modulated and projected to k, v, and pass through unchanged).
    layers: list of dicts of arrays, matrices stored [out_features, in_features]:
         w_mod,b_mod, w_qkv,b_qkv, w_o,b_o, w_up,b_up, w_down,b_down,
         xattn_* (kind 1), 'txt' sub-dict (kind 2).

    Buffer rows: joint-attention kinds store the T text rows first, then the L
    image rows; the other kinds store the L image rows only.

    storage_round: None for the oracle proper (exact float64 everywhere).  A test
    may pass a function (e.g. round-to-nearest-even to bf16): it is then applied
    to every intermediate tensor that a reduced-precision implementation keeps
    in its storage type between two contractions - the normalised and modulated
    rows, q / k / v (after norm and RoPE), the softmax weights, the attention
    output, the GELU output, and for kind 1 the cross-attention's input copy,
    queries, text keys / values and output - and to nothing else (residual
    stream, modulation vectors, statistics and accumulations stay exact).  This
    measures what the storage format alone costs; it is a probe for tolerance
    tests, not a second definition of the stage.
    """

    def __init__(self, cfg, layers, storage_round=None):
        self.cfg = dict(cfg)
        self._sr = storage_round
        self.on_layer = None           # optional callback(layer index) after each block: progress lines of long runs
        self.kind = int(cfg["kind"])
        self.layers = [self._as64(w) for w in layers]
        self.nl = len(self.layers)
        self.d = int(cfg["hidden"])
        self.H = int(cfg["n_heads"])
        self.dh = int(cfg["head_dim"])
        self.F = int(cfg["mlp_dim"])
        self.L = int(cfg["seq_img"])
        self.M = int(cfg["n_patches"])
        self.n = self.L // self.M
        self.T = int(cfg.get("text_len", 0))
        self.Tj = self.T if self.kind in (KIND_MMDIT_JOINT, KIND_SINGLE_STREAM) else 0
        self.Lkv = self.L + self.Tj
        self.eps = float(cfg.get("ln_eps", 1e-6))
        self.theta = float(cfg.get("rope_theta", 1e4))
        self.gelu_tanh = bool(cfg.get("gelu_tanh", 1))
        self.gw = int(cfg["grid_w"])
        self.qk_norm = bool(cfg.get("qk_norm", 0))
        self.joint_rope = bool(cfg.get("joint_rope", 0)) and self.kind == KIND_MMDIT_JOINT
        self.txt_pre_only_last = bool(cfg.get("txt_pre_only_last", 0)) and self.kind == KIND_MMDIT_JOINT
        self.kbuf = [np.zeros((self.Lkv, self.d), F64) for _ in range(self.nl)]
        self.vbuf = [np.zeros((self.Lkv, self.d), F64) for _ in range(self.nl)]
        self.kc = [None] * self.nl     # kind 1: text keys / values of the cross-attention
        self.vc = [None] * self.nl
        self.ready = False

    def _st(self, t):
        """Storage-rounding probe (identity for the oracle proper)."""
        return t if self._sr is None else np.asarray(self._sr(t), F64)

    @staticmethod
    def _as64(w):
        return {k: (StageOracle._as64(v) if isinstance(v, dict) else np.asarray(v, F64)) for k, v in w.items()}

    # -- a0: modulation vectors ------------------------------------------------
    def modulation(self, w, cond):
        """Chunks of width d, order [shift1, scale1, gate1, shift2, scale2, gate2]
        (kind 3: [shift, scale, gate])."""
        cond = np.asarray(cond, F64)
        if self.kind == KIND_ADALN_SINGLE_XATTN:
            m = w["w_mod"].reshape(-1) + cond           # per-layer table + shared 6d vector
        else:
            m = linear(silu(cond), w["w_mod"], w["b_mod"])
        return m.reshape(-1, self.d)

    def _rope(self, t, img_rows):
        """RoPE for rows laid out [text rows ..., image rows ...]; img_rows = global image token
        indices of the image rows (text rows sit at grid position (0,0): no rotation)."""
        n_txt = t.shape[0] - len(img_rows)
        rows = np.concatenate([np.zeros(n_txt), np.asarray(img_rows) // self.gw])
        cols = np.concatenate([np.zeros(n_txt), np.asarray(img_rows) % self.gw])
        return rope_apply(t, rope_angles(rows, cols, self.dh, self.theta), self.H)

    # -- the block stack on a set of rows ---------------------------------------
    def _run(self, x_img, img_off, cond, text):
        """Run all layers on image rows [img_off, img_off+len(x_img)) (and, for the joint kinds,
        on the text rows when `text` is given).  Fresh K/V is written into the buffers before
        each layer's attention (PipeFusion, Sec. 3.3)."""
        kind, d, H = self.kind, self.d, self.H
        x = np.array(x_img, F64)
        n = x.shape[0]
        xt = None
        if kind in (KIND_MMDIT_JOINT, KIND_SINGLE_STREAM) and text is not None:
            xt = np.array(text, F64)
        img_tokens = np.arange(img_off, img_off + n)
        row0 = self.Tj + img_off                         # first buffer row of these image rows

        for l, w in enumerate(self.layers):
            if kind == KIND_SINGLE_STREAM:
                # ---- Flux-like single stream: shared weights on [text; image] rows
                rows = x if xt is None else np.concatenate([xt, x], axis=0)
                nt = 0 if xt is None else xt.shape[0]
                sh, sc, g = self.modulation(w, cond)
                h = self._st(ln_modulate(rows, sh, sc, self.eps))
                qkv = linear(h, w["w_qkv"], w["b_qkv"])
                q, k, v = qkv[:, :d], qkv[:, d:2 * d], qkv[:, 2 * d:]
                if self.qk_norm:
                    q = rms_norm_heads(q, w["q_norm_w"], H, self.eps)
                    k = rms_norm_heads(k, w["k_norm_w"], H, self.eps)
                q = self._st(self._rope(q, img_tokens))
                k = self._st(self._rope(k, img_tokens))
                v = self._st(v)
                if nt:
                    self.kbuf[l][:nt] = k[:nt]
                    self.vbuf[l][:nt] = v[:nt]
                self.kbuf[l][row0:row0 + n] = k[nt:]
                self.vbuf[l][row0:row0 + n] = v[nt:]
                a = self._st(attention(q, self.kbuf[l], self.vbuf[l], H, weight_round=self._sr))
                m = self._st(gelu(linear(h, w["w_up"], w["b_up"]), self.gelu_tanh))
                rows = rows + g * linear(np.concatenate([a, m], axis=1), w["w_down"], w["b_down"])
                if nt:
                    xt, x = rows[:nt], rows[nt:]
                else:
                    x = rows
                if self.on_layer:
                    self.on_layer(l)
                continue

            # ---- kinds 0, 1, 2: sequential attention then MLP
            streams = [(x, w)]
            if kind == KIND_MMDIT_JOINT and xt is not None:
                streams = [(xt, w["txt"]), (x, w)]       # text rows first, own weights
            mods, qs = [], []
            pre_only = self.txt_pre_only_last and l == self.nl - 1      # text stream: keys and values only
            for si, (xs, ws) in enumerate(streams):
                mod = self.modulation(ws, cond)
                mods.append(mod)
                h = self._st(ln_modulate(xs, mod[0], mod[1], self.eps))
                qkv = linear(h, ws["w_qkv"], ws["b_qkv"])
                q, k, v = qkv[:, :d], qkv[:, d:2 * d], qkv[:, 2 * d:]
                is_text = (len(streams) == 2 and si == 0)
                if self.qk_norm:
                    q = rms_norm_heads(q, ws["q_norm_w"], H, self.eps)
                    k = rms_norm_heads(k, ws["k_norm_w"], H, self.eps)
                if self.joint_rope and not is_text:      # text rows sit at grid position (0, 0): no rotation
                    q = self._rope(q, img_tokens)
                    k = self._rope(k, img_tokens)
                q, k, v = self._st(q), self._st(k), self._st(v)
                if is_text:
                    self.kbuf[l][: xs.shape[0]] = k
                    self.vbuf[l][: xs.shape[0]] = v
                else:
                    self.kbuf[l][row0:row0 + n] = k      # write before attend
                    self.vbuf[l][row0:row0 + n] = v
                if not (pre_only and is_text):
                    qs.append(q)
            a_all = self._st(attention(np.concatenate(qs, axis=0), self.kbuf[l], self.vbuf[l], H, weight_round=self._sr))
            new, r = [], 0
            for si, ((xs, ws), mod) in enumerate(zip(streams, mods)):
                if pre_only and len(streams) == 2 and si == 0:
                    new.append(xs)                       # no attention output, no MLP for these rows
                    continue
                a = a_all[r:r + xs.shape[0]]
                r += xs.shape[0]
                xs = xs + mod[2] * linear(a, ws["w_o"], ws["b_o"])
                if kind == KIND_ADALN_SINGLE_XATTN:
                    qc = self._st(linear(self._st(xs), ws["xattn_wq"], ws["xattn_bq"]))
                    ac = self._st(attention(qc, self.kc[l], self.vc[l], H, weight_round=self._sr))
                    xs = xs + linear(ac, ws["xattn_wo"], ws["xattn_bo"])
                h2 = self._st(ln_modulate(xs, mod[3], mod[4], self.eps))
                u = self._st(gelu(linear(h2, ws["w_up"], ws["b_up"]), self.gelu_tanh))
                xs = xs + mod[5] * linear(u, ws["w_down"], ws["b_down"])
                new.append(xs)
            if len(new) == 2:
                xt, x = new
            else:
                x = new[0]
            if self.on_layer:
                self.on_layer(l)
        return x, xt

    # -- warm-up / initialisation of the stale buffers ---------------------------
    def kv_init(self, x_prev=None, cond_prev=None, text=None):
        """Fill the K/V buffers.  With x_prev: one synchronous full-sequence pass (the warm-up
        step of Sec. 3.3).  Without: zeros (App. B).  For kind 1 the text keys/values of the
        cross-attention are computed here once (text does not change across diffusion steps)."""
        if self.kind == KIND_ADALN_SINGLE_XATTN:
            if text is None:
                raise ValueError("kind 1 needs the text features at kv_init")
            for l, w in enumerate(self.layers):
                kv = self._st(linear(text, w["xattn_wkv"], w["xattn_bkv"]))
                self.kc[l], self.vc[l] = kv[:, :self.d], kv[:, self.d:]
        if x_prev is None:
            for l in range(self.nl):
                self.kbuf[l][:] = 0.0
                self.vbuf[l][:] = 0.0
            self.ready = True
            return None
        if self.Tj and text is None:
            raise ValueError("joint kinds need text rows for the warm-up pass")
        self.ready = True
        return self._run(x_prev, 0, cond_prev, text if self.Tj else None)

    def patch_forward(self, x_patch, cond, p, text=None):
        """One stage pass on patch p.  Returns y_patch (and text_out for joint kinds when text rows
        ride along)."""
        if not self.ready:
            raise RuntimeError("kv_init must run first")
        if not (0 <= p < self.M):
            raise IndexError("patch index out of range")
        assert x_patch.shape == (self.n, self.d)
        y, yt = self._run(x_patch, p * self.n, cond, text if self.Tj else None)
        return (y, yt) if (self.Tj and text is not None) else y

    def kv_view(self, layer):
        return self.kbuf[layer], self.vbuf[layer]

    def set_kv(self, layer, k, v):
        self.kbuf[layer][:] = np.asarray(k, F64)
        self.vbuf[layer][:] = np.asarray(v, F64)
        self.ready = True
