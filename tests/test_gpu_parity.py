"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs.  Codes, distances and index arrays must be identical; attention within 2e-3 max-abs."""
import math

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
    # name: config at sizes the oracle finishes in seconds; several tiles and ragged tails
    "c1": C["C1"],
    "c2_ragged": C["C2"].scaled(n_q_heads=4, n_kv_heads=4, n_tokens=9000 + 37, topk=181, needles=5),
    "c4_gqa": C["C4"].scaled(batch=2, n_tokens=5000 + 13, topk=300, needles=3),
    "c5_512": C["C5-512"].scaled(batch=1, n_q_heads=2, n_kv_heads=2, n_tokens=3000 + 5, topk=64, needles=2, extra_tokens=3),
    "lin_128": C["C2"].scaled(n_q_heads=2, n_kv_heads=2, n_tokens=2049, topk=50, hidden=0, needles=2),
    "lin_512_rot": C["C2"].scaled(n_q_heads=2, n_kv_heads=2, n_tokens=4500, topk=90, hidden=0, code_bits=512,
                                  lsh_init="rotation", needles=2),
    "lin_1024_rot": C["C2"].scaled(n_q_heads=2, n_kv_heads=2, n_tokens=4500, topk=90, hidden=0, code_bits=1024,
                                   lsh_init="rotation", needles=2),
    "mlp_1024_g2": C["C2"].scaled(n_q_heads=2, n_kv_heads=1, n_tokens=4097, topk=70, hidden=128, code_bits=1024, needles=2),
    "odd_words": C["C2"].scaled(n_q_heads=2, n_kv_heads=1, n_tokens=1500, topk=33, code_bits=96, hidden=64, needles=2),
    "one_word": C["C1"].scaled(n_tokens=1300, topk=200, code_bits=32, hidden=8, needles=2),
    "f32_kv_bf16_w": C["C1"].scaled(n_tokens=777, topk=77, weight_dtype="bf16", needles=2),
    "g8": C["C4"].scaled(batch=1, n_q_heads=8, n_kv_heads=1, n_tokens=4200, topk=100, code_bits=128, hidden=256, needles=1),
    # more query + key vectors per step than compute units: the hash kernel that serves several
    # vectors of one weight head per workgroup (full tiles; ragged last tiles; the linear hash)
    "many_vectors": C["C4"].scaled(batch=20, n_q_heads=16, n_kv_heads=4, n_tokens=700 + 3, topk=90, hidden=128,
                                   code_bits=128, needles=1),
    "many_vectors_ragged": C["C4"].scaled(batch=7, n_q_heads=40, n_kv_heads=20, n_tokens=500 + 9, topk=80, hidden=128,
                                          code_bits=64, needles=1),
    "many_vectors_lin": C["C4"].scaled(batch=9, n_q_heads=32, n_kv_heads=16, n_tokens=400 + 1, topk=75, hidden=0,
                                       code_bits=128, needles=1),
}


@pytest.fixture(scope="module", params=sorted(SMALL))
def case(request):
    c = Case(SMALL[request.param])
    yield c
    c.close()


def test_generator_is_identical_on_host_and_device():
    w = wl.Workload(C["C2"].scaled(n_q_heads=2, n_kv_heads=2, n_tokens=5000))
    for which in ("K", "V"):
        a = w.kv_rows(which, 0, 1, 100, 3000, "cpu")
        b = w.kv_rows(which, 0, 1, 100, 3000, "cuda:0").cpu()
        assert torch.equal(a, b)
    assert torch.equal(w.synthetic_codes(0, 1, 7, 500, "cpu"), w.synthetic_codes(0, 1, 7, 500, "cuda:0").cpu())
    for a, b in zip(w.hash_weights("cpu"), w.hash_weights("cuda:0")):
        assert torch.equal(a, b.cpu())


def test_hash_keys_bit_exact(case):
    cfg = case.cfg
    case.codes.fill_(0x3C3C3C3C)
    case.ctx.hash_keys(case.K, *case.weights, 0, cfg.n_tokens, case.codes)
    want = case.oracle_codes()
    got = case.codes.cpu()
    assert torch.equal(got[:, :, :cfg.n_tokens], want[:, :, :cfg.n_tokens])
    if cfg.max_tokens > cfg.n_tokens:
        assert (got[:, :, cfg.n_tokens:] == 0x3C3C3C3C).all()     # rows outside the range untouched


def test_hash_append_one_key(case):
    """Decode-step append: one new key per head at t0, every other row untouched."""
    cfg = case.cfg
    t0 = cfg.n_tokens - 1
    case.codes.fill_(0x11111111)
    case.ctx.hash_keys(case.K, *case.weights, t0, 1, case.codes)
    want = torch.full_like(case.codes.cpu(), 0x11111111)
    oracle.hash_keys(case.hK, *case.hweights, cfg.code_bits, t0, 1, want)
    assert torch.equal(case.codes.cpu(), want)
    # a short run of rows takes the 8-row tile path
    case.codes.fill_(0x11111111)
    n = min(13, cfg.n_tokens)
    case.ctx.hash_keys(case.K, *case.weights, 2, n, case.codes)
    want = torch.full_like(want, 0x11111111)
    oracle.hash_keys(case.hK, *case.hweights, cfg.code_bits, 2, n, want)
    assert torch.equal(case.codes.cpu(), want)


def test_retrieve_bit_exact_from_oracle_codes(case):
    """Retrieval alone: both sides start from the oracle's key codes."""
    cfg = case.cfg
    hcodes = case.oracle_codes()
    dcodes = hcodes.to(case.dev)
    B, Hq, N, k = cfg.batch, cfg.n_q_heads, cfg.n_tokens, cfg.topk
    qcode = torch.empty(B, Hq, cfg.words, dtype=torch.int32, device=case.dev)
    dist = torch.empty(B, Hq, N, dtype=torch.int16, device=case.dev)
    idx = case.ctx.retrieve_topk(case.q, *case.weights, dcodes, N, k, out_qcode=qcode, out_dist=dist)
    widx, wq, wdist = oracle.retrieve_topk(case.w.q, *case.hweights, hcodes, N, k, want_dist=True)
    assert torch.equal(qcode.cpu(), wq)
    assert torch.equal(dist.cpu(), wdist)
    assert torch.equal(idx.cpu(), widx)
    # planted needles are retrieved
    for b in range(B):
        for hq in range(Hq):
            assert set(case.w.needle_pos[b, hq].tolist()) <= set(idx[b, hq].tolist())


@pytest.mark.parametrize("kind", ["k1", "kN", "short_context"])
def test_retrieve_edge_k(case, kind):
    cfg = case.cfg
    hcodes = case.oracle_codes()
    dcodes = hcodes.to(case.dev)
    N = cfg.n_tokens
    if kind == "k1":
        n, k = N, 1
    elif kind == "kN":
        n, k = N, N
    else:
        n, k = 129, 17      # far fewer tokens than the capacity; a single partial block
    idx = case.ctx.retrieve_topk(case.q, *case.weights, dcodes, n, k)
    widx, _, _ = oracle.retrieve_topk(case.w.q, *case.hweights, hcodes, n, k)
    assert torch.equal(idx.cpu(), widx)
    if kind == "kN":
        assert torch.equal(idx[0, 0].cpu(), torch.arange(N, dtype=torch.int32))


def test_sparse_decode_within_tolerance(case):
    cfg = case.cfg
    hcodes = case.oracle_codes()
    widx, _, _ = oracle.retrieve_topk(case.w.q, *case.hweights, hcodes, cfg.n_tokens, cfg.topk)
    want = oracle.sparse_decode(case.w.q, case.hK, case.hV, widx, case.scale)
    got = case.ctx.sparse_decode(case.q, case.K, case.V, widx.to(case.dev), case.scale).cpu()
    assert float((got - want).abs().max()) <= ATTN_TOL
    # k = N: full attention over the cache (Eq. 1)
    n = cfg.n_tokens
    full = torch.arange(n, dtype=torch.int32).expand(cfg.batch, cfg.n_q_heads, n).contiguous()
    want = oracle.sparse_decode(case.w.q, case.hK, case.hV, full, case.scale)
    got = case.ctx.sparse_decode(case.q, case.K, case.V, full.to(case.dev), case.scale).cpu()
    assert float((got - want).abs().max()) <= ATTN_TOL
    # a single row returns that value row; order of idx does not matter
    one = torch.full((cfg.batch, cfg.n_q_heads, 1), 5, dtype=torch.int32)
    got = case.ctx.sparse_decode(case.q, case.K, case.V, one.to(case.dev), case.scale).cpu()
    G = cfg.group
    for b in range(cfg.batch):
        for hq in range(cfg.n_q_heads):
            assert torch.equal(got[b, hq], case.hV[b, hq // G, 5].float())
    perm = widx[:, :, torch.randperm(cfg.topk, generator=torch.Generator().manual_seed(1))].contiguous()
    got_p = case.ctx.sparse_decode(case.q, case.K, case.V, perm.to(case.dev), case.scale).cpu()
    want = oracle.sparse_decode(case.w.q, case.hK, case.hV, widx, case.scale)
    assert float((got_p - want).abs().max()) <= ATTN_TOL


def test_full_chain_matches_oracle_chain(case):
    """hash -> retrieve -> attend entirely on the GPU against the same chain in the oracle."""
    cfg = case.cfg
    case.codes.zero_()
    case.ctx.hash_keys(case.K, *case.weights, 0, cfg.n_tokens, case.codes)
    idx = case.ctx.retrieve_topk(case.q, *case.weights, case.codes, cfg.n_tokens, cfg.topk)
    out = case.ctx.sparse_decode(case.q, case.K, case.V, idx, case.scale)
    hcodes = case.oracle_codes()
    widx, _, _ = oracle.retrieve_topk(case.w.q, *case.hweights, hcodes, cfg.n_tokens, cfg.topk)
    want = oracle.sparse_decode(case.w.q, case.hK, case.hV, widx, case.scale)
    assert torch.equal(idx.cpu(), widx)
    assert float((out.cpu() - want).abs().max()) <= ATTN_TOL
    # same call twice: identical bits (no atomics on any output path)
    idx2 = case.ctx.retrieve_topk(case.q, *case.weights, case.codes, cfg.n_tokens, cfg.topk)
    out2 = case.ctx.sparse_decode(case.q, case.K, case.V, idx2, case.scale)
    assert torch.equal(idx, idx2) and torch.equal(out, out2)


def test_ties_resolved_towards_lower_index():
    """Degenerate code caches: all keys equal (every distance ties) and two-level distances."""
    cfg = C["C2"].scaled(n_q_heads=2, n_kv_heads=2, n_tokens=10000, topk=1234, needles=0)
    c = Case(cfg)
    try:
        codes = torch.zeros(1, 2, cfg.max_tokens, cfg.words, dtype=torch.int32)
        codes[:, :, 5000:] = -1           # second half: all bits set
        codes[:, 1, 7] = 0x0F0F0F0F
        dcodes = codes.to(c.dev)
        for k in (1, 1234, 5000, 5001, 9999, 10000):
            idx = c.ctx.retrieve_topk(c.q, *c.weights, dcodes, cfg.n_tokens, k)
            widx, _, _ = oracle.retrieve_topk(c.w.q, *c.hweights, codes, cfg.n_tokens, k)
            assert torch.equal(idx.cpu(), widx), k
    finally:
        c.close()


def test_out_of_range_indices_are_skipped():
    cfg = C["C2"].scaled(n_q_heads=2, n_kv_heads=2, n_tokens=600, topk=40, needles=0)
    c = Case(cfg)
    try:
        good = torch.arange(0, 80, 2, dtype=torch.int32).expand(1, 2, 40).contiguous()
        bad = good.clone()
        bad[:, :, 3] = -1
        bad[:, :, 17] = cfg.max_tokens
        keep = torch.ones(40, dtype=torch.bool)
        keep[3] = keep[17] = False
        want = oracle.sparse_decode(c.w.q, c.hK, c.hV, good[:, :, keep].contiguous(), c.scale)
        got = c.ctx.sparse_decode(c.q, c.K, c.V, bad.to(c.dev), c.scale).cpu()
        assert float((got - want).abs().max()) <= ATTN_TOL
    finally:
        c.close()


def test_bulk_hash_on_matrix_cores_equals_the_binary32_kernel_and_the_oracle():
    """Bulk hashing runs its second layer on the matrix cores and recomputes outputs too close to
    zero with the defined binary32 chain.  Rows built to stress that: zeros (every output exactly
    0: the whole tile goes to the recomputation), tiny and huge magnitudes, a NaN and an infinity."""
    import paper_2508_19740_amd as sp
    cfg = C["C2"].scaled(n_q_heads=2, n_kv_heads=2, n_tokens=40000 + 19, topk=64, needles=0)
    c = Case(cfg)
    try:
        K = c.K
        K[0, 0, 64:160] = 0                                   # three tiles of zero rows
        K[0, 1, 1000:1040] *= 1e-30
        K[0, 1, 2000:2040] *= 1e18
        K[0, 0, 3000, 5] = float("nan")
        K[0, 1, 3001, 7] = float("inf")
        c.hK = K.cpu()
        n = cfg.n_tokens
        c.codes.fill_(0)
        c.ctx.hash_keys(K, *c.weights, 0, n, c.codes)         # matrix-core path (bf16 weights, hidden 256)
        got = c.codes.clone()
        c.ctx.set_option(sp.OPT_BULK_HASH_MATRIX_CORES, 0)
        try:
            c.codes.fill_(0)
            c.ctx.hash_keys(K, *c.weights, 0, n, c.codes)     # all-binary32 kernel
        finally:
            c.ctx.set_option(sp.OPT_BULK_HASH_MATRIX_CORES, 1)
        assert torch.equal(got, c.codes)
        # the same call audited: every output also evaluated with the chain, inside the kernel
        c.ctx.set_option(sp.OPT_BULK_HASH_AUDIT, 1)
        c.codes.fill_(0)
        c.ctx.hash_keys(K, *c.weights, 0, n, c.codes)
        c.ctx.set_option(sp.OPT_BULK_HASH_AUDIT, 0)
        au = c.ctx.bulk_hash_audit_read()
        assert torch.equal(got, c.codes)
        assert au["outputs"] == 2 * n * cfg.code_bits and au["wrong"] == 0
        assert 0 < au["listed"] < au["outputs"] // 50
        assert 0.0 < au["max_ratio"] < au["eps"]
        want = c.oracle_codes(0, 6000)                        # the stressed rows and their surroundings
        assert torch.equal(got.cpu()[:, :, :6000], want[:, :, :6000])
        # a second layer of zeros for head 0: every output is exactly 0, no sign can be certified, every
        # tile of that head overflows its list and is recomputed whole
        w1, b1, w2 = (t.clone() for t in c.weights)
        w2[0] = 0
        c.codes.fill_(-1)
        c.ctx.hash_keys(K, w1, b1, w2, 0, n, c.codes)
        assert int(c.codes[:, 0, :n].abs().max()) == 0       # sign(0) is bit 0
        hw = tuple(t.cpu() for t in (w1, b1, w2))
        want2 = torch.zeros_like(want)
        oracle.hash_keys(c.hK, *hw, cfg.code_bits, 0, 3000, want2)
        assert torch.equal(c.codes.cpu()[:, :, :3000], want2[:, :, :3000])
    finally:
        c.close()
