"""Shared helpers of the GPU parity tests: build one workload on the device and on the host."""
from __future__ import annotations

import math

import torch

import oracle
import workload as wl


def torch_dtype(name):
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


class Case:
    """Device tensors of one Config plus (optionally) the oracle's results on host copies."""

    def __init__(self, cfg: wl.Config, device="cuda:0", host_copy=True, max_topk=None):
        import paper_2508_19740_amd as sp

        self.cfg = cfg
        self.dev = torch.device(device)
        self.w = wl.Workload(cfg)
        self.K = self.w.materialize("K", self.dev)
        self.V = self.w.materialize("V", self.dev)
        self.q = self.w.q.to(self.dev)
        self.weights = tuple(None if t is None else t.to(self.dev) for t in self.w.hash_weights())
        self.codes = torch.zeros(cfg.batch, cfg.n_kv_heads, cfg.max_tokens, cfg.words,
                                 dtype=torch.int32, device=self.dev)
        if max_topk is None:
            max_topk = cfg.max_tokens if cfg.max_tokens <= 65536 else cfg.topk
        self.ctx = sp.Spotlight(cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.code_bits, cfg.hidden,
                                cfg.max_tokens, max_topk,
                                kv_dtype=torch_dtype(cfg.kv_dtype), weight_dtype=torch_dtype(cfg.weight_dtype),
                                device=self.dev)
        self.scale = 1.0 / math.sqrt(cfg.head_dim)
        if host_copy:
            self.hK = self.K.cpu()
            self.hV = self.V.cpu()
            self.hweights = self.w.hash_weights()

    # oracle on the host copies -------------------------------------------------------------
    def oracle_codes(self, t0=0, n=None):
        cfg = self.cfg
        n = cfg.n_tokens if n is None else n
        codes = torch.zeros(cfg.batch, cfg.n_kv_heads, cfg.max_tokens, cfg.words, dtype=torch.int32)
        oracle.hash_keys(self.hK, *self.hweights, cfg.code_bits, t0, n, codes)
        return codes

    def step_path(self, one_launch: bool):
        """Which way spotlight_decode_step runs a short context: one kernel, or the five of the general path."""
        import paper_2508_19740_amd as sp
        self.ctx.set_option(sp.OPT_STEP_SINGLE_LAUNCH, 1 if one_launch else 0)

    def launches_of(self, fn):
        """Kernel launches per stage that fn() makes on this context."""
        self.ctx.profile_enable(True)
        try:
            fn()
            return {name: n for name, (_, n) in self.ctx.profile_read().items()}
        finally:
            self.ctx.profile_enable(False)

    def close(self):
        self.ctx.close()
