"""The PipeFusion sampling loop (Sec. 3.3) run on ONE device: N stage objects chained, M patches, S steps.

Host orchestration only: every arithmetic step is a library call (pf_kv_init, pf_stage_patch_forward, pf_op_axpy).
On N devices, device i would hold stage i and run item k = (step, patch) at micro-step k + i; a stage's K/V buffer only
changes through its own calls, which arrive in the order of k, so running the items back to back here gives the same
values as the N-device schedule (only the P2P transfers between stages are missing).
"""
from __future__ import annotations

import torch

from .binding import Stage, pf_op_axpby, pf_op_axpy


class Pipeline:
    """stage_layers: one list of layer-weight dicts per stage.  All tensors passed in live on the device:
    x [L, d] float32, cond float32, joint-kind text rows float32, kind-1 text features in the stage dtype."""

    def __init__(self, cfg, stage_layers, kernel_path=0, device="cuda"):
        self.cfg = dict(cfg)
        self.stages = [Stage(cfg, layers, kernel_path=kernel_path, device=device) for layers in stage_layers]
        self.N = len(self.stages)
        self.M = int(cfg["n_patches"])
        self.L = int(cfg["seq_img"])
        self.n = self.L // self.M
        self.d = int(cfg["hidden"])
        self.joint = int(cfg["kind"]) in (2, 3)
        f32 = dict(dtype=torch.float32, device=device)
        # ping-pong hidden-state rows between consecutive stages (what P2P would carry), allocated once
        self._h = [torch.empty(self.n, self.d, **f32) for _ in range(2)]
        T = int(cfg.get("text_len", 0)) if self.joint else 0
        self._t = [torch.empty(T, self.d, **f32) for _ in range(2)] if T else None
        self.eps = torch.empty(self.L, self.d, **f32)

    def warmup_step(self, x, cond, text=None):
        """Synchronous step (Sec. 3.3 warm-up): full sequence through every stage; fills every K/V buffer.  Returns eps."""
        h, ht = x, text
        for st in self.stages:
            if self.joint:
                h, ht = st.kv_init(h, cond, ht, want_output=True)
            else:
                h, _ = st.kv_init(h, cond, text, want_output=True)
        self.eps.copy_(h)
        return self.eps

    def pipelined_step(self, x, cond, text=None):
        """One step after warm-up.  eps rows of patch p are written straight into self.eps by the last stage.  The
        timestep embedding is the same for all M patches of the step: every stage derives its modulation vectors on
        patch 0 and keeps them for the rest."""
        n = self.n
        for p in range(self.M):
            src = x[p * n:(p + 1) * n]
            tsrc = text if (self.joint and p == 0 and text is not None) else None
            for i, st in enumerate(self.stages):
                dst = self.eps[p * n:(p + 1) * n] if i == self.N - 1 else self._h[i & 1]
                if tsrc is not None:
                    st.patch_forward(src, cond, p, text=tsrc, out=dst, text_out=self._t[i & 1], same_cond=p > 0)
                    tsrc = self._t[i & 1]
                else:
                    st.patch_forward(src, cond, p, out=dst, same_cond=p > 0)
                src = dst
        return self.eps

    def run(self, x_T, conds, dts, warmup_steps=1, text=None):
        """S = len(conds) steps, the first `warmup_steps` synchronous; Euler update x += dt * eps after each (Sec. 2, Eq. 1).
        Returns x_0 (a new tensor; x_T is left untouched)."""
        x = x_T.clone()
        for s, (c, dt) in enumerate(zip(conds, dts)):
            eps = self.warmup_step(x, c, text) if s < warmup_steps else self.pipelined_step(x, c, text)
            pf_op_axpy(x, eps, dt, out=x)
        return x

    def destroy(self):
        for st in self.stages:
            st.destroy()


class CfgPipeline:
    """The sampling loop with classifier-free guidance on one device: the conditional and the unconditional pass of a
    step share every call (stages created with batch = 2: image 0 conditional, image 1 unconditional, same latent),
    eps = eps_u + scale * (eps_c - eps_u) is one pf_op_axpby, the update one pf_op_axpy.
    conds: per step a [2, ...] tensor (conditional, unconditional); text likewise [2, T, ...] or None."""

    def __init__(self, cfg, stage_layers, kernel_path=0, device="cuda"):
        self.cfg = dict(cfg, batch=2)
        self.stages = [Stage(self.cfg, layers, kernel_path=kernel_path, device=device) for layers in stage_layers]
        self.N = len(self.stages)
        self.M = int(cfg["n_patches"])
        self.L = int(cfg["seq_img"])
        self.n = self.L // self.M
        self.d = int(cfg["hidden"])
        self.joint = int(cfg["kind"]) in (2, 3)
        f32 = dict(dtype=torch.float32, device=device)
        self._in = torch.empty(2, self.n, self.d, **f32)                      # the patch of both images (same rows twice)
        self._h = [torch.empty(2, self.n, self.d, **f32) for _ in range(2)]   # hand-over between consecutive stages
        T = int(cfg.get("text_len", 0)) if self.joint else 0
        self._t = [torch.empty(2, T, self.d, **f32) for _ in range(2)] if T else None
        self.eps2 = torch.empty(2, self.L, self.d, **f32)
        self.eps = torch.empty(self.L, self.d, **f32)
        self._x2 = torch.empty(2, self.L, self.d, **f32)

    def _combine(self, scale):
        pf_op_axpby(self.eps2[1], self.eps2[0], 1.0 - scale, scale, out=self.eps)
        return self.eps

    def warmup_step(self, x, cond2, scale, text2=None):
        self._x2[0].copy_(x)
        self._x2[1].copy_(x)
        h, ht = self._x2, text2
        for st in self.stages:
            if self.joint:
                h, ht = st.kv_init(h, cond2, ht, want_output=True)
            else:
                h, _ = st.kv_init(h, cond2, text2, want_output=True)
        self.eps2.copy_(h)
        return self._combine(scale)

    def pipelined_step(self, x, cond2, scale, text2=None):
        n = self.n
        for p in range(self.M):
            self._in[0].copy_(x[p * n:(p + 1) * n])
            self._in[1].copy_(x[p * n:(p + 1) * n])
            src = self._in
            tsrc = text2 if (self.joint and p == 0 and text2 is not None) else None
            for i, st in enumerate(self.stages):
                dst = self._h[i & 1]
                if tsrc is not None:
                    st.patch_forward(src, cond2, p, text=tsrc, out=dst, text_out=self._t[i & 1], same_cond=p > 0)
                    tsrc = self._t[i & 1]
                else:
                    st.patch_forward(src, cond2, p, out=dst, same_cond=p > 0)
                src = dst
            self.eps2[:, p * n:(p + 1) * n].copy_(src)
        return self._combine(scale)

    def run(self, x_T, conds2, dts, scale, warmup_steps=1, text2=None):
        x = x_T.clone()
        for s, (c2, dt) in enumerate(zip(conds2, dts)):
            eps = self.warmup_step(x, c2, scale, text2) if s < warmup_steps else self.pipelined_step(x, c2, scale, text2)
            pf_op_axpy(x, eps, dt, out=x)
        return x

    def destroy(self):
        for st in self.stages:
            st.destroy()
