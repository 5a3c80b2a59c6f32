"""GPU parity of the one-call decode step (appended-key hash + query hash in one launch, retrieval
with forced sink / local tokens, attention) against the oracle's decode step."""
import numpy as np
import pytest
import torch

import oracle
import workload as wl
from gpu_common import Case

pytestmark = pytest.mark.gpu
ATTN_TOL = 2e-3

C = wl.CONFIGS
SMALL = {
    "c1": C["C1"],
    "c2_ragged": C["C2"].scaled(n_q_heads=4, n_kv_heads=4, n_tokens=9000 + 37, topk=181, needles=5),
    "c4_gqa": C["C4"].scaled(batch=2, n_tokens=5000 + 13, topk=300, needles=3),
    "c5_512": C["C5-512"].scaled(batch=1, n_q_heads=2, n_kv_heads=2, n_tokens=3000 + 5, topk=100, needles=2, extra_tokens=3),
    "lin_128": C["C2"].scaled(n_q_heads=2, n_kv_heads=2, n_tokens=2049, topk=90, hidden=0, needles=2),
    "odd_words": C["C2"].scaled(n_q_heads=2, n_kv_heads=1, n_tokens=1500, topk=133, code_bits=96, hidden=64, needles=2),
    "lin_1024_rot": C["C2"].scaled(n_q_heads=2, n_kv_heads=2, n_tokens=4500, topk=90, hidden=0, code_bits=1024,
                                   lsh_init="rotation", needles=2),
    "block_edge": C["C2"].scaled(n_q_heads=2, n_kv_heads=2, n_tokens=3 * 4096, topk=200, needles=2),
    "g8": C["C4"].scaled(batch=1, n_q_heads=8, n_kv_heads=1, n_tokens=4200, topk=100, code_bits=128, hidden=256, needles=1),
    # more query + key vectors per step than compute units: the hash kernel that serves several
    # vectors of one weight head per workgroup (full tiles; ragged last tiles; the linear hash)
    "many_vectors": C["C4"].scaled(batch=20, n_q_heads=16, n_kv_heads=4, n_tokens=700 + 3, topk=90, hidden=128,
                                   code_bits=128, needles=1),
    "many_vectors_ragged": C["C4"].scaled(batch=7, n_q_heads=40, n_kv_heads=20, n_tokens=500 + 9, topk=80, hidden=128,
                                          code_bits=64, needles=1),
    "many_vectors_lin": C["C4"].scaled(batch=9, n_q_heads=32, n_kv_heads=16, n_tokens=400 + 1, topk=75, hidden=0,
                                       code_bits=128, needles=1),
    # 28 query heads on 4 key-value heads (groups of seven), the head layout of Qwen2.5-7B
    "g7": C["C4"].scaled(batch=1, n_q_heads=28, n_kv_heads=4, n_tokens=6000 + 7, topk=150, code_bits=128, hidden=256, needles=1),
    # the two mixed pairings of key / value and weight element types
    "f32_kv_bf16_w": C["C1"].scaled(n_tokens=777, topk=77, weight_dtype="bf16", needles=2),
    "bf16_kv_f32_w": C["C2"].scaled(n_q_heads=2, n_kv_heads=2, n_tokens=1900, topk=90, weight_dtype="f32", needles=2),
    # contexts that take three and four bitmap words per thread in the single-launch step (its longest)
    "long_40k": C["C2"].scaled(n_q_heads=2, n_kv_heads=1, n_tokens=40000 + 19, topk=800, hidden=128, needles=2),
    "long_64k": C["C2"].scaled(n_q_heads=1, n_kv_heads=1, n_tokens=65536, topk=1311, hidden=128, code_bits=64, needles=2),
}
FORCED = [(0, 0), (4, 64), (0, 1), (7, 0)]
# cases the single-launch step serves (codes of at most 256 bits, hidden width a multiple of 128):
# they run both ways, as one kernel and as the five kernels of the general path
ONE_LAUNCH = {"c1", "c2_ragged", "c4_gqa", "lin_128", "block_edge", "g8", "many_vectors", "many_vectors_ragged",
              "many_vectors_lin", "long_40k", "long_64k", "f32_kv_bf16_w", "bf16_kv_f32_w", "g7"}
PARAMS = [(name, False) for name in sorted(SMALL)] + [(name, True) for name in sorted(ONE_LAUNCH)]


@pytest.fixture(scope="module", params=PARAMS, ids=[f"{n}-{'one_launch' if o else 'five_launches'}" for n, o in PARAMS])
def case(request):
    name, one_launch = request.param
    c = Case(SMALL[name])
    c.one_launch = one_launch
    c.step_path(one_launch)
    cfg = c.cfg
    # code cache of all tokens but the last, by the oracle (no oracle input comes from the GPU)
    c.base_codes = c.oracle_codes(0, cfg.n_tokens - 1)
    yield c
    c.close()


def test_the_step_takes_the_path_it_is_tested_on(case):
    cfg = case.cfg
    case.codes.copy_(case.base_codes)
    ran = case.launches_of(lambda: case.ctx.decode_step(case.q, case.K, case.V, *case.weights, case.codes,
                                                         cfg.n_tokens, cfg.topk, 4, 8))
    if case.one_launch:
        assert ran["step_small"] == 1 and ran["score"] == ran["hash_query"] == ran["attend"] == 0
    else:
        assert ran["step_small"] == 0 and ran["score"] == ran["select"] == ran["attend"] == ran["merge"] == 1


@pytest.mark.parametrize("forced", FORCED)
def test_decode_step_matches_oracle(case, forced):
    cfg = case.cfg
    n_sink, n_local = forced
    n = cfg.n_tokens
    want_codes = case.base_codes.clone()
    want_idx, want_out = oracle.decode_step(case.w.q, case.hK, case.hV, *case.hweights, want_codes, n, cfg.topk,
                                            n_sink, n_local, case.scale)
    case.codes.copy_(case.base_codes)
    idx, out = case.ctx.decode_step(case.q, case.K, case.V, *case.weights, case.codes, n, cfg.topk, n_sink, n_local)
    assert torch.equal(case.codes.cpu(), want_codes)                 # the appended key's code, nothing else
    assert torch.equal(idx.cpu(), want_idx)
    assert float((out.cpu() - want_out).abs().max()) <= ATTN_TOL
    if n_sink or n_local:
        got = idx.cpu()
        for t in list(range(n_sink)) + list(range(n - n_local, n)):
            assert (got == t).any(dim=-1).all()


def test_forced_tokens_across_block_borders(case):
    """Sink and local windows longer than a 4096-token block, and windows that meet."""
    cfg = case.cfg
    n = cfg.n_tokens
    for n_sink, n_local, k in ((min(n // 3, 4100), min(n // 3, 4200), min(n, 2 * (n // 3) + 40)),
                               (n // 2, n - n // 2, n), (n, n, n)):
        want_codes = case.base_codes.clone()
        want_idx, _ = oracle.decode_step(case.w.q, case.hK, case.hV, *case.hweights, want_codes, n, k,
                                         n_sink, n_local, case.scale)
        case.codes.copy_(case.base_codes)
        idx, _ = case.ctx.decode_step(case.q, case.K, case.V, *case.weights, case.codes, n, k, n_sink, n_local)
        assert torch.equal(idx.cpu(), want_idx), (n_sink, n_local, k)


def test_step_without_forced_tokens_equals_the_three_calls(case):
    cfg = case.cfg
    n = cfg.n_tokens
    case.codes.copy_(case.base_codes)
    idx, out = case.ctx.decode_step(case.q, case.K, case.V, *case.weights, case.codes, n, cfg.topk)
    c2 = case.base_codes.to(case.dev)
    case.ctx.hash_keys(case.K, *case.weights, n - 1, 1, c2)
    idx2 = case.ctx.retrieve_topk(case.q, *case.weights, c2, n, cfg.topk)
    out2 = case.ctx.sparse_decode(case.q, case.K, case.V, idx2)
    assert torch.equal(case.codes, c2)
    assert torch.equal(idx, idx2)
    if case.one_launch:     # same rows, another order of summation
        assert float((out - out2).abs().max()) <= ATTN_TOL
    else:
        assert torch.equal(out, out2)


def test_prepacked_weights_change_nothing_but_the_load_order(case):
    """With the packed copy of the weights in the workspace, the decode step, the retrieval alone
    and the one-key append give the oracle's codes and indices, and the same attention output."""
    cfg = case.cfg
    n = cfg.n_tokens
    want_codes = case.base_codes.clone()
    want_idx, want_out = oracle.decode_step(case.w.q, case.hK, case.hV, *case.hweights, want_codes, n, cfg.topk,
                                            4, 64, case.scale)
    case.codes.copy_(case.base_codes)
    _, out_plain = case.ctx.decode_step(case.q, case.K, case.V, *case.weights, case.codes, n, cfg.topk, 4, 64)
    case.ctx.prepack_weights(*case.weights)
    try:
        case.codes.copy_(case.base_codes)
        idx, out = case.ctx.decode_step(case.q, case.K, case.V, *case.weights, case.codes, n, cfg.topk, 4, 64)
        assert torch.equal(case.codes.cpu(), want_codes)
        assert torch.equal(idx.cpu(), want_idx)
        assert float((out.cpu() - want_out).abs().max()) <= ATTN_TOL
        assert torch.equal(out, out_plain)
        # the single calls read the copy as well
        qcode = torch.empty(cfg.batch, cfg.n_q_heads, cfg.words, dtype=torch.int32, device=case.dev)
        idx2 = case.ctx.retrieve_topk(case.q, *case.weights, case.codes, n, cfg.topk, out_qcode=qcode)
        widx, wq, _ = oracle.retrieve_topk(case.w.q, *case.hweights, want_codes, n, cfg.topk)
        assert torch.equal(qcode.cpu(), wq)
        assert torch.equal(idx2.cpu(), widx)
        case.codes.copy_(case.base_codes)
        case.ctx.hash_keys(case.K, *case.weights, n - 1, 1, case.codes)
        assert torch.equal(case.codes.cpu(), want_codes)
    finally:
        case.ctx.prepack_weights()   # dropped: the other tests read the arrays themselves


def test_prepacked_copy_serves_only_the_arrays_it_was_made_from():
    """The copy is a snapshot keyed by the three pointers: other arrays are read directly, and
    after a change in place the copy has to be made again."""
    cfg = C["C2"].scaled(n_q_heads=4, n_kv_heads=2, n_tokens=300, topk=20, needles=1)
    c = Case(cfg)
    try:
        t0 = cfg.n_tokens - 1

        def oracle_row(hweights):
            want = torch.zeros(cfg.batch, cfg.n_kv_heads, cfg.max_tokens, cfg.words, dtype=torch.int32)
            oracle.hash_keys(c.hK, *hweights, cfg.code_bits, t0, 1, want)
            return want

        w1, b1, w2 = c.weights
        hw1, hb1, hw2 = c.hweights
        c.ctx.prepack_weights(w1, b1, w2)
        # other arrays (every output's sign flipped): their own contents count, not the copy
        w2_neg = (-w2).contiguous()
        c.codes.zero_()
        c.ctx.hash_keys(c.K, w1, b1, w2_neg, t0, 1, c.codes)
        want_neg = oracle_row((hw1, hb1, -hw2))
        assert torch.equal(c.codes.cpu(), want_neg)
        assert not torch.equal(want_neg, oracle_row((hw1, hb1, hw2)))
        # changed in place and packed again
        w2.neg_()
        c.ctx.prepack_weights(w1, b1, w2)
        c.codes.zero_()
        c.ctx.hash_keys(c.K, w1, b1, w2, t0, 1, c.codes)
        assert torch.equal(c.codes.cpu(), want_neg)
        # dropped: back to the arrays
        c.ctx.prepack_weights()
        w2.neg_()
        c.codes.zero_()
        c.ctx.hash_keys(c.K, w1, b1, w2, t0, 1, c.codes)
        assert torch.equal(c.codes.cpu(), oracle_row((hw1, hb1, hw2)))
    finally:
        c.close()


def test_decode_step_rejects_bad_arguments(case):
    import paper_2508_19740_amd as sp
    cfg = case.cfg
    n = cfg.n_tokens
    args = (case.q, case.K, case.V, *case.weights, case.codes)
    for kw in (dict(n_tokens=n, k=10, n_sink=8, n_local=3),       # 11 forced tokens, k = 10
               dict(n_tokens=n, k=10, n_sink=-1, n_local=0),
               dict(n_tokens=n, k=10, n_sink=0, n_local=-2),
               dict(n_tokens=0, k=1, n_sink=0, n_local=0),
               dict(n_tokens=cfg.max_tokens + 1, k=1, n_sink=0, n_local=0),
               dict(n_tokens=n, k=n + 1, n_sink=0, n_local=0)):
        with pytest.raises(sp.SpotlightError) as e:
            case.ctx.decode_step(*args, kw["n_tokens"], kw["k"], kw["n_sink"], kw["n_local"])
        assert e.value.rc == sp.ERR_INVALID_ARG


@pytest.mark.parametrize("one_launch", [False, True])
def test_decode_step_in_a_hip_graph(one_launch):
    """The call is kernel launches (five, or one) and nothing else, so it can be captured.  Replayed
    several times with eager work and synchronisations in between; every replay equals the eager result."""
    cfg = C["C2"].scaled(n_q_heads=4, n_kv_heads=4, n_tokens=9000 + 37, topk=181, needles=5)
    c = Case(cfg)
    c.step_path(one_launch)
    try:
        n = cfg.n_tokens
        base = c.oracle_codes(0, n - 1).to(c.dev)
        c.codes.copy_(base)
        idx_e, out_e = c.ctx.decode_step(c.q, c.K, c.V, *c.weights, c.codes, n, cfg.topk, 4, 64)
        codes_e = c.codes.clone()
        torch.cuda.synchronize()
        idx_g = torch.empty_like(idx_e)
        out_g = torch.empty_like(out_e)
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        c.codes.copy_(base)
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            graph.capture_begin()
            c.ctx.decode_step(c.q, c.K, c.V, *c.weights, c.codes, n, cfg.topk, 4, 64, out_idx=idx_g, out=out_g)
            graph.capture_end()
        torch.cuda.synchronize()
        for rep in range(4):
            c.codes.copy_(base)
            idx_g.fill_(-7)
            out_g.fill_(float("nan"))
            junk = (torch.randn(1 << 20, device=c.dev) * (rep + 1)).sum()     # eager work between replays
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.isfinite(junk)
            assert torch.equal(c.codes, codes_e), rep
            assert torch.equal(idx_g, idx_e), rep
            assert torch.equal(out_g, out_e), rep
    finally:
        c.close()
