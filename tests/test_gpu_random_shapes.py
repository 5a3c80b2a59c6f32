"""GPU parity over seeded random shapes: batch, heads, group size, code length, hidden width, context
length, k and forced windows drawn at random inside what the library supports, each run through the
one-call decode step (general path, and the single-launch path where it applies) and through the
three separate calls, against the oracle."""
import random

import pytest
import torch

import oracle
import workload as wl
from gpu_common import Case

pytestmark = pytest.mark.gpu
ATTN_TOL = 2e-3


def draw(seed):
    r = random.Random(seed)
    group = r.choice([1, 1, 2, 3, 4, 5, 6, 7, 8])
    n_kv = r.choice([1, 2, 3, 5])
    words = r.choice([1, 2, 3, 4, 4, 5, 7, 8, 8, 12, 16, 32]) if group <= 2 else r.choice([1, 2, 4, 4, 6, 8, 8, 11, 16])
    hidden = r.choice([0, 8, 64, 128, 128, 256, 384])
    n = r.choice([1, 2, 63, 64, 65, 255, 1000, 4095, 4096, 4097, 8191, 9000, 12288, 20000])
    k = max(1, min(n, r.choice([1, 2, 7, 64, n // 50 + 1, n // 7 + 1, n])))
    n_sink = r.choice([0, 0, 1, 4, 100])
    n_local = r.choice([0, 0, 1, 64, 300])
    if min(n, n_sink + n_local) > k:
        n_sink, n_local = 0, min(n_local, k) if r.random() < 0.5 else 0
    kv = r.choice(["bf16", "bf16", "f32"])
    wd = r.choice(["bf16", "bf16", "f32"])
    cfg = wl.CONFIGS["C2"].scaled(batch=r.choice([1, 1, 2, 3]), n_q_heads=n_kv * group, n_kv_heads=n_kv, n_tokens=n,
                                  topk=k, hidden=hidden, code_bits=32 * words, kv_dtype=kv, weight_dtype=wd,
                                  needles=min(2, max(0, n // (4 * group))), seed=31337 + seed,
                                  extra_tokens=r.choice([0, 0, 5]))
    return cfg, n_sink, n_local


@pytest.mark.parametrize("seed", range(160))
def test_random_shape_matches_the_oracle(seed):
    cfg, n_sink, n_local = draw(seed)
    n, k = cfg.n_tokens, cfg.topk
    c = Case(cfg, max_topk=k)
    try:
        base = c.oracle_codes(0, n - 1) if n > 1 else torch.zeros(cfg.batch, cfg.n_kv_heads, cfg.max_tokens, cfg.words,
                                                                  dtype=torch.int32)
        want_codes = base.clone()
        want_idx, want_out = oracle.decode_step(c.w.q, c.hK, c.hV, *c.hweights, want_codes, n, k, n_sink, n_local, c.scale)
        small_ok = cfg.words <= 8 and cfg.hidden % 128 == 0
        for one_launch in ((False, True) if small_ok else (False,)):
            c.step_path(one_launch)
            c.codes.copy_(base)
            idx, out = c.ctx.decode_step(c.q, c.K, c.V, *c.weights, c.codes, n, k, n_sink, n_local)
            assert torch.equal(c.codes.cpu(), want_codes), (one_launch, cfg)
            assert torch.equal(idx.cpu(), want_idx), (one_launch, cfg)
            assert float((out.cpu() - want_out).abs().max()) <= ATTN_TOL, (one_launch, cfg)
        if n_sink == 0 and n_local == 0:
            # the three calls: bulk hash of the whole cache (every row), retrieval with distances, attention
            c.codes.zero_()
            c.ctx.hash_keys(c.K, *c.weights, 0, n, c.codes)
            assert torch.equal(c.codes.cpu()[:, :, :n], want_codes[:, :, :n]), cfg
            dist = torch.empty(cfg.batch, cfg.n_q_heads, n, dtype=torch.int16, device=c.dev)
            qcode = torch.empty(cfg.batch, cfg.n_q_heads, cfg.words, dtype=torch.int32, device=c.dev)
            idx3 = c.ctx.retrieve_topk(c.q, *c.weights, c.codes, n, k, out_qcode=qcode, out_dist=dist)
            widx, wq, wdist = oracle.retrieve_topk(c.w.q, *c.hweights, want_codes, n, k, want_dist=True)
            assert torch.equal(qcode.cpu(), wq) and torch.equal(dist.cpu(), wdist) and torch.equal(idx3.cpu(), widx), cfg
            out3 = c.ctx.sparse_decode(c.q, c.K, c.V, idx3, c.scale)
            assert float((out3.cpu() - want_out).abs().max()) <= ATTN_TOL, cfg
    finally:
        c.close()
