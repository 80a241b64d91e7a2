"""CPU oracle for the whole PipeFusion sampling loop on one device: N stage oracles chained, M patches, S steps.

TEST INFRASTRUCTURE ONLY (same rules as pf_oracle.py: imported by tests, the smoke check and benchmark baselines;
never by the product path; shares no code with the HIP library).

What the paper fixes:
  * Sec. 2, Eq. 1: one diffusion step is x_{t-1} = Update(x_t, t, eps(x_t, t, c)), element-wise in the latent once the
    network output is known.  The update used here is the Euler form x_{t-1} = x_t + dt_t * eps, dt_t given by the caller
    (the sampler itself is not part of the method; any element-wise rule works patch by patch).
  * Sec. 3.3: the first step(s) are warm-up steps: synchronous, the whole sequence goes through every stage, no stale
    activations; they also leave the full-sequence K/V in every stage's buffer.
  * Sec. 3.3: afterwards patch p of step t passes stage 0 .. N-1; each stage writes the patch's fresh K/V into its buffer
    and attends over the buffer whose other rows come from patches 0..p-1 of this step and from the previous step.  As
    soon as the last stage finishes patch p, the update gives patch p of x_{t-1}, which re-enters stage 0 for step t-1.
  * Sec. 3.3 / Fig. 4: on N devices, device i works on item k = (step, patch) at micro-step k + i.  A stage's buffer
    only changes through its own calls, which come in the order of k on every device, so running the items one after the
    other on one device (for step, for patch, for stage) gives exactly the values of the N-device schedule.  The test suite
    checks this with a micro-step-ordered emulation.
  * Sec. 3.4: the time of one image is (M*S + N - 1) micro-steps for M*S items, so the fraction of busy device time is
    M*S / (M*S + N - 1).

Reading: the network output eps is taken to be the hidden state after the last stage (patch embedding, final layer and
unpatchify are outside the stage stack and identical with or without PipeFusion).
"""
from __future__ import annotations

import numpy as np

from .pf_oracle import StageOracle

F64 = np.float64


def euler_update(x, eps, dt):
    """x_{t-1} = x_t + dt * eps (Sec. 2, Eq. 1 with an Euler rule)."""
    return np.asarray(x, F64) + float(dt) * np.asarray(eps, F64)


def pipeline_utilisation(M, S, N):
    """Busy fraction of the N devices over one image: M*S items, each device idle for N-1 micro-steps (Sec. 3.4)."""
    return (M * S) / float(M * S + N - 1)


class PipelineOracle:
    """stage_layers: list (one entry per stage) of lists of layer-weight dicts.  cfg as for StageOracle."""

    def __init__(self, cfg, stage_layers):
        self.cfg = dict(cfg)
        self.stages = [StageOracle(cfg, layers) for layers in stage_layers]
        self.N = len(self.stages)
        self.M = int(cfg["n_patches"])
        self.L = int(cfg["seq_img"])
        self.n = self.L // self.M
        self.joint = int(cfg["kind"]) in (2, 3)

    def warmup_step(self, x, cond, text=None):
        """Synchronous step: full sequence through every stage, K/V buffers filled on the way.  Returns eps [L, d]."""
        h, ht = np.asarray(x, F64), (None if text is None else np.asarray(text, F64))
        for st in self.stages:
            if self.joint:
                h, ht = st.kv_init(h, cond, ht)
            else:
                h, _ = st.kv_init(h, cond, text)       # kind 1: text = encoder features for the cross-attention
        return h

    def pipelined_step(self, x, cond, text=None):
        """One step after warm-up: patches one after the other, each through all stages.  Returns eps [L, d]."""
        eps = np.zeros((self.L, x.shape[1]), F64)
        for p in range(self.M):
            h = np.asarray(x[p * self.n:(p + 1) * self.n], F64)
            ht = np.asarray(text, F64) if (self.joint and p == 0 and text is not None) else None
            for st in self.stages:
                if ht is not None:
                    h, ht = st.patch_forward(h, cond, p, text=ht)   # the text rows ride with patch 0
                else:
                    h = st.patch_forward(h, cond, p)
            eps[p * self.n:(p + 1) * self.n] = h
        return eps

    def run(self, x_T, conds, dts, warmup_steps=1, text=None):
        """S = len(conds) steps; the first `warmup_steps` are synchronous.  Returns (x_0, [eps of every step])."""
        x = np.array(x_T, F64)
        trace = []
        for s, (c, dt) in enumerate(zip(conds, dts)):
            eps = self.warmup_step(x, c, text) if s < warmup_steps else self.pipelined_step(x, c, text)
            trace.append(eps)
            x = euler_update(x, eps, dt)
        return x, trace


# --------------------------------------------------------------------------- #
# cost model of the parallel schemes (Sec. 3.4, Table 1)                       #
# --------------------------------------------------------------------------- #
def scheme_costs(scheme, p, hs, L, N, kv_bytes_per_layer, param_bytes):
    """Per-device cost of one diffusion step as the table of Sec. 3.4 states it (orders of magnitude, constants as
    printed): communicated elements, whether the communication overlaps with compute, parameter bytes and K/V
    activation bytes held.  p = sequence length, hs = hidden size, L = layers, N = devices;
    kv_bytes_per_layer = bytes of full-sequence K and V of one layer."""
    KV = kv_bytes_per_layer
    rows = {
        "tensor_parallel": (4 * p * hs * L, False, param_bytes / N, KV / N),
        "distrifusion":    (2 * p * hs * L, True, param_bytes, KV * L),
        "sp_ring":         (2 * p * hs * L, True, param_bytes, KV / N),
        "sp_ulysses":      (4 * p * hs * L / N, False, param_bytes, KV / N),
        "pipefusion":      (2 * p * hs, True, param_bytes / N, KV * L / N),
    }
    comm, overlap, params, kv = rows[scheme]
    return {"comm_elements": comm, "overlap": overlap, "param_bytes": params, "kv_bytes": kv}


class CfgPipelineOracle:
    """Classifier-free guidance on top of the patch pipeline: every step runs the stage stack on the same latent with
    the conditional and the unconditional conditioning (two independent sets of K/V buffers, shared weights; the paper
    runs the two on separate device groups, Sec. 4.1, CFG parallel), combines eps = eps_u + scale * (eps_c - eps_u) and applies
    the update."""

    def __init__(self, cfg, stage_layers):
        self.cond_pipe = PipelineOracle(cfg, stage_layers)
        self.uncond_pipe = PipelineOracle(cfg, stage_layers)

    def run(self, x_T, conds_c, conds_u, dts, scale, warmup_steps=1, text_c=None, text_u=None):
        x = np.array(x_T, F64)
        trace = []
        for s, (cc, cu, dt) in enumerate(zip(conds_c, conds_u, dts)):
            if s < warmup_steps:
                ec, eu = self.cond_pipe.warmup_step(x, cc, text_c), self.uncond_pipe.warmup_step(x, cu, text_u)
            else:
                ec, eu = self.cond_pipe.pipelined_step(x, cc, text_c), self.uncond_pipe.pipelined_step(x, cu, text_u)
            eps = eu + float(scale) * (ec - eu)
            trace.append(eps)
            x = euler_update(x, eps, dt)
        return x, trace
