"""spotlight_decode_step_noalloc (the decode step for callers that cannot allocate: its workspace is
a fixed buffer inside the library) against spotlight_decode_step on a context, through the C ABI:
two calls in a row, the second on a smaller problem whose buffers land elsewhere in the shared
scratch, so that whatever the first call left behind must not matter."""
import ctypes as C
import math

import pytest
import torch

import workload as wl
from gpu_common import Case

pytestmark = pytest.mark.gpu
ATTN_TOL = 2e-3

BIG = wl.CONFIGS["C2"].scaled(n_q_heads=8, n_kv_heads=4, n_tokens=3 * 4096 + 57, topk=400, needles=3, extra_tokens=2)
SMALL = wl.CONFIGS["C2"].scaled(n_q_heads=2, n_kv_heads=2, n_tokens=4096 + 901, topk=77, needles=2, seed=991, extra_tokens=1)


def _both_ways(cfg, n_sink, n_local):
    """(idx, out, codes) of the context's entry point and of the one without allocation."""
    import paper_2508_19740_amd as sp
    c = Case(cfg, host_copy=False, max_topk=cfg.topk)
    try:
        n, k = cfg.n_tokens, cfg.topk
        c.ctx.hash_keys(c.K, *c.weights, 0, n - 1, c.codes)            # the cache before the step; row n-1 is the step's
        codes_ctx, codes_na = c.codes.clone(), c.codes.clone()
        idx_ctx, out_ctx = c.ctx.decode_step(c.q, c.K, c.V, *c.weights, codes_ctx, n, k, n_sink, n_local)
        idx_na = torch.full_like(idx_ctx, -1)
        out_na = torch.full_like(out_ctx, float("nan"))
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        rc = sp.spotlight_decode_step_noalloc(c.ctx.cfg, c.q, c.K, c.V, *c.weights, codes_na, n, k, n_sink, n_local,
                                              c.scale, idx_na, out_na)
        assert rc == sp.OK, rc
        assert torch.cuda.memory_allocated() == before
        torch.cuda.synchronize()
        return (idx_ctx.cpu(), out_ctx.cpu(), codes_ctx.cpu()), (idx_na.cpu(), out_na.cpu(), codes_na.cpu())
    finally:
        c.close()


def test_step_without_allocation_equals_the_step_on_a_context():
    for cfg, n_sink, n_local in ((BIG, 4, 64), (SMALL, 0, 0)):
        (idx_a, out_a, codes_a), (idx_b, out_b, codes_b) = _both_ways(cfg, n_sink, n_local)
        assert torch.equal(codes_a, codes_b), cfg.name                  # the appended key's code
        assert int(codes_a[:, :, cfg.n_tokens - 1].abs().max()) != 0
        assert torch.equal(idx_a, idx_b), cfg.name
        assert float((out_a - out_b).abs().max()) <= ATTN_TOL, cfg.name
        assert bool(torch.isfinite(out_b).all())


def test_shapes_beyond_the_fixed_buffer_are_refused():
    import paper_2508_19740_amd as sp
    c4 = wl.CONFIGS["C4"]
    cfg = sp.make_config(c4.batch, c4.n_q_heads, c4.n_kv_heads, c4.code_bits, c4.hidden, c4.max_tokens, c4.topk)
    assert sp.workspace_bytes(cfg) > sp.NOALLOC_SCRATCH_BYTES
    t = torch.zeros(64, dtype=torch.int32, device="cuda:0")           # never read: the refusal comes first
    rc = sp.lib.spotlight_decode_step_noalloc(C.byref(cfg), t.data_ptr(), t.data_ptr(), t.data_ptr(),
                                              C.byref(sp.HashWeights(t.data_ptr(), t.data_ptr(), t.data_ptr())),
                                              t.data_ptr(), 1000, 10, 0, 0, 1.0 / math.sqrt(128), t.data_ptr(), t.data_ptr())
    assert rc == sp.ERR_TOO_LARGE
