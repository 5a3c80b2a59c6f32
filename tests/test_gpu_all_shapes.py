"""GPU parity over every supported (code length, heads per group) pair (17 code lengths x groups of 1 to 8): each pair is its own
instantiation of the score and select kernels (lanes per key, histogram replicas, batch sizes and
register budgets all depend on it), so each one runs the one-call decode step against the oracle:
appended code, index arrays (with and without forced tokens) bit-exact, attention within 2e-3."""
import pytest
import torch

import oracle
import workload as wl
from gpu_common import Case

pytestmark = pytest.mark.gpu
ATTN_TOL = 2e-3

WORDS = list(range(1, 17)) + [32]
PAIRS = [(w, g) for w in WORDS for g in range(1, 9) if not (w == 32 and g > 2)]


@pytest.mark.parametrize("words,group", PAIRS)
def test_decode_step_for_every_code_length_and_group_size(words, group):
    # two full 4096-token blocks and a ragged third; linear hash (the oracle's cost stays small);
    # few distinct distances at short codes, so ties cross block borders
    n = 2 * 4096 + 37 * words + group
    cfg = wl.CONFIGS["C2"].scaled(batch=1, n_q_heads=group, n_kv_heads=1, n_tokens=n, topk=64 + 5 * words,
                                  hidden=0, code_bits=32 * words, needles=2, seed=900 + 17 * words + group)
    c = Case(cfg)
    try:
        base = c.oracle_codes(0, n - 1)
        # the general path (its kernels are what this test instantiates), then, for codes of at most
        # 256 bits, the same step as one kernel launch
        for one_launch in ((False, True) if words <= 8 else (False,)):
            c.step_path(one_launch)
            for n_sink, n_local, k in ((0, 0, cfg.topk), (4, 64, cfg.topk), (0, 1, 1), (3, 0, n // 2)):
                want_codes = base.clone()
                want_idx, want_out = oracle.decode_step(c.w.q, c.hK, c.hV, *c.hweights, want_codes, n, k,
                                                        n_sink, n_local, c.scale)
                c.codes.copy_(base)
                idx, out = c.ctx.decode_step(c.q, c.K, c.V, *c.weights, c.codes, n, k, n_sink, n_local)
                assert torch.equal(c.codes.cpu(), want_codes), (one_launch, n_sink, n_local, k)
                assert torch.equal(idx.cpu(), want_idx), (one_launch, n_sink, n_local, k)
                assert float((out.cpu() - want_out).abs().max()) <= ATTN_TOL, (one_launch, n_sink, n_local, k)
            ran = c.launches_of(lambda: c.ctx.decode_step(c.q, c.K, c.V, *c.weights, c.codes, n, cfg.topk, 0, 0))
            assert (ran["step_small"], ran["score"]) == ((1, 0) if one_launch else (0, 1))
    finally:
        c.close()
