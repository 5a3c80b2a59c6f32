"""Pins for the oracle's forced-token top-k and its one-call decode step (CPU only).

Forced tokens are the "Sink" and "Local" columns of the paper's perplexity comparison with
MagicPIG (first 4, last 64 tokens kept next to the retrieved ones); the current token that Eq. 1
concatenates is a local window of one.
"""
import math

import numpy as np
import pytest
import torch

import oracle
import workload as wl


def _lexsort_forced(dist, k, n_sink, n_local):
    """One sort with 'not forced' as the leading key: a different formulation from the oracle's
    (which sets the forced tokens aside first and sorts only the others)."""
    n = len(dist)
    t = np.arange(n)
    forced = (t < n_sink) | (t >= n - n_local)
    order = np.lexsort((t, dist, ~forced))   # last key is the primary one
    return np.sort(order[:k]).astype(np.int32)


def test_forced_topk_hand_worked():
    # tokens 0..7 with these distances; sink 1 -> {0}; local 2 -> {6, 7}; one more: the nearest of
    # tokens 1..5 is token 5 (distance 0)
    d = torch.tensor([5, 1, 9, 1, 7, 0, 3, 8], dtype=torch.int16)
    assert oracle.topk_forced(d, 4, 1, 2).tolist() == [0, 5, 6, 7]
    # two more: tokens 1 and 3 tie at distance 1, the lower index goes first
    assert oracle.topk_forced(d, 5, 1, 2).tolist() == [0, 1, 5, 6, 7]
    assert oracle.topk_forced(d, 6, 1, 2).tolist() == [0, 1, 3, 5, 6, 7]
    # a forced token is kept however far it is: token 2 (distance 9) as part of a sink of 3
    assert oracle.topk_forced(d, 4, 3, 0).tolist() == [0, 1, 2, 5]
    # exactly the forced set
    assert oracle.topk_forced(d, 3, 1, 2).tolist() == [0, 6, 7]


def test_forced_topk_without_forced_tokens_is_topk():
    for seed in range(5):
        n = 300 + 17 * seed
        d = wl.uniform_int(seed, 9, 0, n, 12).to(torch.int16)
        for k in (1, 7, n // 2, n):
            assert torch.equal(oracle.topk_forced(d, k, 0, 0), oracle.topk(d, k))


@pytest.mark.parametrize("seed", range(6))
def test_forced_topk_matches_single_lexsort(seed):
    n = 64 + 29 * seed
    d = wl.uniform_int(seed, 11, 0, n, 6).to(torch.int16)     # few values: many ties
    for n_sink, n_local in ((0, 1), (4, 0), (4, 8), (1, 1), (3, 20)):
        for k in (n_sink + n_local, n_sink + n_local + 1, n // 2, n):
            got = oracle.topk_forced(d, k, n_sink, n_local).numpy()
            assert np.array_equal(got, _lexsort_forced(d.numpy(), k, n_sink, n_local)), (n_sink, n_local, k)


def test_forced_topk_overlap_and_errors():
    d = torch.tensor([3, 2, 1, 0], dtype=torch.int16)
    # sink and local windows overlap: the forced set is all four tokens, counted once
    assert oracle.topk_forced(d, 4, 3, 3).tolist() == [0, 1, 2, 3]
    with pytest.raises(ValueError):
        oracle.topk_forced(d, 3, 3, 3)        # more forced tokens than k
    with pytest.raises(ValueError):
        oracle.topk_forced(d, 2, 2, 1)
    with pytest.raises(ValueError):
        oracle.topk_forced(d, 2, -1, 0)


def _setup(cfg):
    w = wl.Workload(cfg)
    w1, b1, w2 = w.hash_weights()
    K = w.materialize("K", "cpu")
    V = w.materialize("V", "cpu")
    codes = torch.zeros(cfg.batch, cfg.n_kv_heads, cfg.max_tokens, cfg.words, dtype=torch.int32)
    oracle.hash_keys(K, w1, b1, w2, cfg.code_bits, 0, cfg.n_tokens - 1, codes)   # all but the new token
    return w, w1, b1, w2, K, V, codes


def test_decode_step_is_the_chain_of_the_single_calls():
    cfg = wl.CONFIGS["C4"].scaled(batch=2, n_q_heads=4, n_kv_heads=2, n_tokens=300, topk=24,
                                  hidden=64, code_bits=64, needles=2)
    w, w1, b1, w2, K, V, codes = _setup(cfg)
    scale = 1.0 / math.sqrt(cfg.head_dim)
    n = cfg.n_tokens
    c_step = codes.clone()
    idx, out = oracle.decode_step(w.q, K, V, w1, b1, w2, c_step, n, cfg.topk, 4, 8, scale)
    # the new key's code has been appended, nothing else touched
    c_ref = codes.clone()
    oracle.hash_keys(K, w1, b1, w2, cfg.code_bits, n - 1, 1, c_ref)
    assert torch.equal(c_step, c_ref)
    assert not torch.equal(c_step[:, :, n - 1], codes[:, :, n - 1])
    _, _, dist = oracle.retrieve_topk(w.q, w1, b1, w2, c_ref, n, cfg.topk, want_dist=True)
    for b in range(cfg.batch):
        for hq in range(cfg.n_q_heads):
            hk = hq // cfg.group
            want = _lexsort_forced(dist[b, hq].numpy(), cfg.topk, 4, 8)
            assert np.array_equal(idx[b, hq].numpy(), want)
            assert set(range(4)) | set(range(n - 8, n)) <= set(idx[b, hq].tolist())
            o = oracle.sparse_attention(w.q[b, hq].contiguous(), K[b, hk], V[b, hk], idx[b, hq].contiguous(), scale)
            assert torch.equal(out[b, hq], o)


def test_decode_step_special_cases():
    cfg = wl.CONFIGS["C1"].scaled(n_tokens=257, topk=32, needles=4)
    w, w1, b1, w2, K, V, codes = _setup(cfg)
    scale = 1.0 / math.sqrt(cfg.head_dim)
    n = cfg.n_tokens
    # no forced tokens: the plain retrieve + attend
    c0 = codes.clone()
    idx0, out0 = oracle.decode_step(w.q, K, V, w1, b1, w2, c0, n, cfg.topk, 0, 0, scale)
    idx_p, _, _ = oracle.retrieve_topk(w.q, w1, b1, w2, c0, n, cfg.topk)
    assert torch.equal(idx0, idx_p)
    assert torch.equal(out0, oracle.sparse_decode(w.q, K, V, idx_p, scale))
    # local window of one = the current token of Eq. 1 is always attended
    c1 = codes.clone()
    idx1, _ = oracle.decode_step(w.q, K, V, w1, b1, w2, c1, n, cfg.topk, 0, 1, scale)
    assert int(idx1[0, 0, -1]) == n - 1
    # k = N: forced tokens change nothing, the result is full attention over the cache (Eq. 1)
    c2 = codes.clone()
    idx2, out2 = oracle.decode_step(w.q, K, V, w1, b1, w2, c2, n, n, 4, 64, scale)
    assert idx2[0, 0].tolist() == list(range(n))
    s = (K[0, 0, :n].double() @ w.q[0, 0].double()) * scale
    p = torch.softmax(s, dim=0)
    want = (p[:, None] * V[0, 0, :n].double()).sum(0)
    assert float((out2[0, 0].double() - want).abs().max()) < 1e-6
