"""Exact full-sequence forward of a stack of DiT blocks, written with torch.nn.functional
library routines in float64.  It knows nothing about patches, K/V buffers or staleness: it
is the "original model" that PipeFusion (Sec. 3.3) must reproduce when M = 1 or when the
buffer is fresh everywhere, and serves as an independent pin for the oracle.

Deliberately a different formulation from the oracle: batched heads through
scaled_dot_product_attention, F.layer_norm, F.gelu, and RoPE via complex multiplication.
"""
import math

import torch
import torch.nn.functional as Fn

DT = torch.float64


def _t(a):
    return torch.as_tensor(a, dtype=DT)


def _mha(q, k, v, H):
    nq, d = q.shape
    dh = d // H
    qh = q.view(nq, H, dh).transpose(0, 1)
    kh = k.view(k.shape[0], H, dh).transpose(0, 1)
    vh = v.view(v.shape[0], H, dh).transpose(0, 1)
    o = Fn.scaled_dot_product_attention(qh, kh, vh)          # default scale 1/sqrt(dh)
    return o.transpose(0, 1).reshape(nq, d)


def _rope_complex(t, grid_rc, H, theta):
    """grid_rc: [n, 2] (row, col) per token.  First half of the head's channels <- row, second <- col."""
    n, d = t.shape
    dh = d // H
    w = dh // 2
    inv = theta ** (-torch.arange(0, w, 2, dtype=DT) / w)                    # [w/2]
    ang = torch.cat([grid_rc[:, :1] * inv, grid_rc[:, 1:] * inv], dim=1)      # [n, dh/2]
    rot = torch.polar(torch.ones_like(ang), ang)                              # e^{i ang}
    tc = torch.view_as_complex(t.reshape(n, H, dh // 2, 2).contiguous())
    return torch.view_as_real(tc * rot[:, None, :]).reshape(n, d)


def _qk_norm(t, w, H, eps):
    n, d = t.shape
    return Fn.rms_norm(t.view(n, H, d // H), (d // H,), weight=_t(w), eps=eps).reshape(n, d)


def _mod(kind, w, cond):
    if kind == 1:
        return (_t(w["w_mod"]).reshape(-1) + cond).view(6, -1)
    m = Fn.linear(Fn.silu(cond), _t(w["w_mod"]), _t(w["b_mod"]))
    return m.view(-1, cond.shape[0])


def full_forward(cfg, layers, x, cond, text=None):
    """Returns (y_img [L,d], y_text or None)."""
    kind, d, H = cfg["kind"], cfg["hidden"], cfg["n_heads"]
    eps = cfg.get("ln_eps", 1e-6)
    approx = "tanh" if cfg.get("gelu_tanh", 1) else "none"
    x = _t(x).clone()
    cond = _t(cond)
    L = x.shape[0]
    xt = _t(text).clone() if (kind in (2, 3) and text is not None) else None
    ln = lambda z: Fn.layer_norm(z, (d,), eps=eps)

    for li, w in enumerate(layers):
        pre_only = bool(cfg.get("txt_pre_only_last")) and kind == 2 and li == len(layers) - 1
        if kind == 3:
            T = xt.shape[0]
            rows = torch.cat([xt, x], 0)
            sh, sc, g = _mod(kind, w, cond)
            h = ln(rows) * (1 + sc) + sh
            q, k, v = Fn.linear(h, _t(w["w_qkv"]), _t(w["b_qkv"])).split(d, dim=1)
            idx = torch.arange(L)
            rc = torch.cat([torch.zeros(T, 2, dtype=DT),
                            torch.stack([idx // cfg["grid_w"], idx % cfg["grid_w"]], 1).to(DT)], 0)
            if cfg.get("qk_norm"):
                q, k = _qk_norm(q, w["q_norm_w"], H, eps), _qk_norm(k, w["k_norm_w"], H, eps)
            q = _rope_complex(q, rc, H, cfg.get("rope_theta", 1e4))
            k = _rope_complex(k, rc, H, cfg.get("rope_theta", 1e4))
            a = _mha(q, k, v, H)
            m = Fn.gelu(Fn.linear(h, _t(w["w_up"]), _t(w["b_up"])), approximate=approx)
            rows = rows + g * Fn.linear(torch.cat([a, m], 1), _t(w["w_down"]), _t(w["b_down"]))
            xt, x = rows[:T], rows[T:]
            continue

        streams = [(x, w)] if kind != 2 else [(xt, w["txt"]), (x, w)]
        mods = [_mod(kind, ws, cond) for _, ws in streams]
        qkvs = []
        for (xs, ws), m in zip(streams, mods):
            h = ln(xs) * (1 + m[1]) + m[0]
            qkvs.append(Fn.linear(h, _t(ws["w_qkv"]), _t(ws["b_qkv"])))
        if cfg.get("qk_norm"):
            qkvs = [torch.cat([_qk_norm(t[:, :d], ws["q_norm_w"], H, eps), _qk_norm(t[:, d:2 * d], ws["k_norm_w"], H, eps),
                               t[:, 2 * d:]], 1) for t, (_, ws) in zip(qkvs, streams)]
        qkv = torch.cat(qkvs, 0)
        qq, kk = qkv[:, :d], qkv[:, d:2 * d]
        if kind == 2 and cfg.get("joint_rope"):
            T = xt.shape[0]
            idx = torch.arange(L)
            rc = torch.cat([torch.zeros(T, 2, dtype=DT),
                            torch.stack([idx // cfg["grid_w"], idx % cfg["grid_w"]], 1).to(DT)], 0)
            qq = _rope_complex(qq.contiguous(), rc, H, cfg.get("rope_theta", 1e4))
            kk = _rope_complex(kk.contiguous(), rc, H, cfg.get("rope_theta", 1e4))
        if pre_only:
            # final joint block: only the image rows are queries; the text rows pass through
            a_img = _mha(qq[xt.shape[0]:], kk, qkv[:, 2 * d:], H)
            a_all = torch.cat([torch.zeros(xt.shape[0], d, dtype=DT), a_img], 0)
        else:
            a_all = _mha(qq, kk, qkv[:, 2 * d:], H)
        outs, r = [], 0
        for si, ((xs, ws), m) in enumerate(zip(streams, mods)):
            if pre_only and si == 0:
                outs.append(xs)
                r += xs.shape[0]
                continue
            a = a_all[r:r + xs.shape[0]]
            r += xs.shape[0]
            xs = xs + m[2] * Fn.linear(a, _t(ws["w_o"]), _t(ws["b_o"]))
            if kind == 1:
                qc = Fn.linear(xs, _t(ws["xattn_wq"]), _t(ws["xattn_bq"]))
                kc, vc = Fn.linear(_t(text), _t(ws["xattn_wkv"]), _t(ws["xattn_bkv"])).split(d, dim=1)
                xs = xs + Fn.linear(_mha(qc, kc, vc, H), _t(ws["xattn_wo"]), _t(ws["xattn_bo"]))
            h2 = ln(xs) * (1 + m[4]) + m[3]
            u = Fn.gelu(Fn.linear(h2, _t(ws["w_up"]), _t(ws["b_up"])), approximate=approx)
            xs = xs + m[5] * Fn.linear(u, _t(ws["w_down"]), _t(ws["b_down"]))
            outs.append(xs)
        if kind == 2:
            xt, x = outs
        else:
            x = outs[0]
    return x.numpy(), (None if xt is None else xt.numpy())
