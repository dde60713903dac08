"""Set a workload from :mod:`rsd_inputs` up on the GPU: weights generated on
the device, prompts and uniforms uploaded, context created.  Plumbing only."""
from __future__ import annotations

import numpy as np

from rsd_inputs import Workload, model_blob_torch, prompt_lengths, prompt_tokens, uniforms

from . import binding as R


class Session:
    """A context plus the device buffers it borrows."""

    def __init__(self, w: Workload, delta=None, weights=None, use_graphs: int = 1, kv_pool_bytes=(0, 0, 0),
                 omega_kind=None, omega_a=None, merge_prm: int = 0, sd_k: int = 0):
        """``merge_prm`` = 1 / 2: the reward head sits on the draft's / target's trunk.  ``w.prm`` must then
        repeat that model's shape; of the reward model's generated blob only the projection (its last
        d_model + 8 elements: w_r, b_r) is handed over."""
        import torch

        self.w = w
        dev = torch.device("cuda:0")
        self.weights = weights if weights is not None else [model_blob_torch(w.seed, i, s, dev) for i, s in enumerate(w.shapes)]
        if merge_prm and weights is None:
            self.weights[2] = self.weights[2][-(w.prm.d_model + 8):].clone()
        self.ctx = R.rsd_init(w.shapes, self.weights, batch=w.batch, merge_prm=merge_prm, delta=w.delta if delta is None else delta,
                              sep_id=w.sep_id, step_cap=w.step_cap, max_steps=w.max_steps, max_ctx=w.max_ctx,
                              eos_id=w.eos_id, temperature=w.temperature, top_p=w.top_p,
                              sep_logit_bias=w.sep_logit_bias,
                              omega_kind=w.omega_kind if omega_kind is None else omega_kind,
                              omega_a=w.omega_a if omega_a is None else omega_a,
                              kv_pool_bytes=kv_pool_bytes, use_graphs=use_graphs, sd_k=sd_k)
        self.prompt_len = prompt_lengths(w)
        self.tokens_host = prompt_tokens(w)
        self.tokens = torch.from_numpy(self.tokens_host).to(dev)
        self.u_host = {k: uniforms(w, k, n) for k, n in (("U_DRAFT", w.max_ctx), ("U_TARGET", w.max_ctx), ("U_GATE", w.max_steps))}
        self.u = {k: torch.from_numpy(v).to(dev) for k, v in self.u_host.items()}
        R.rsd_set_uniforms(self.ctx, self.u["U_DRAFT"], self.u["U_TARGET"], self.u["U_GATE"])
        if sd_k and w.temperature > 0:
            for k in ("U_PROP", "U_ACC"):
                self.u_host[k] = uniforms(w, k, w.max_ctx)
                self.u[k] = torch.from_numpy(self.u_host[k]).to(dev)
            R.rsd_set_uniforms_sd(self.ctx, self.u["U_PROP"], self.u["U_ACC"])
        self.reset()

    def reset(self):
        R.rsd_set_prompts(self.ctx, self.tokens, self.prompt_len)

    def close(self):
        R.rsd_destroy(self.ctx)


class BonSession:
    """A process Best-of-N context: ``w.batch`` sequences x ``n`` candidate lanes, base model = the
    workload's draft model, its reward model; candidate ``k`` of sequence ``s`` draws with row
    ``s * n + k`` of the U_DRAFT stream generated for ``w.batch * n`` rows."""

    def __init__(self, w: Workload, n: int, weights=None, use_graphs: int = 1, kv_pool_bytes=(0, 0, 0)):
        import torch
        from dataclasses import replace

        self.w, self.n = w, n
        dev = torch.device("cuda:0")
        self.weights = weights if weights is not None else [model_blob_torch(w.seed, 0, w.draft, dev), None,
                                                            model_blob_torch(w.seed, 2, w.prm, dev)]
        self.ctx = R.rsd_init(w.shapes, self.weights, batch=w.batch * n, bon_n=n, delta=0.0, sep_id=w.sep_id,
                              step_cap=w.step_cap, max_steps=w.max_steps, max_ctx=w.max_ctx, eos_id=w.eos_id,
                              temperature=w.temperature, top_p=w.top_p, sep_logit_bias=w.sep_logit_bias,
                              kv_pool_bytes=kv_pool_bytes, use_graphs=use_graphs)
        self.prompt_len = prompt_lengths(w)
        self.tokens_host = prompt_tokens(w)
        self.tokens = torch.from_numpy(self.tokens_host).to(dev)
        self.u_host = uniforms(replace(w, batch=w.batch * n), "U_DRAFT", w.max_ctx)      # [batch * n, max_ctx]
        self.u = torch.from_numpy(self.u_host).to(dev)
        R.rsd_set_uniforms(self.ctx, self.u, None, None)
        self.reset()

    def reset(self):
        R.rsd_set_prompts(self.ctx, self.tokens, self.prompt_len)

    def close(self):
        R.rsd_destroy(self.ctx)
