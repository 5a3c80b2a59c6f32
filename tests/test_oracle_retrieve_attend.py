"""Pins for the oracle's Hamming scoring, top-k selection and sparse attention (CPU only)."""
import math

import numpy as np
import pytest
import torch

import oracle
import workload as wl


def _rand_codes(seed, n, W):
    b = wl.random_bits32(seed, 77, 0, n * W).view(n, W)
    return torch.where(b >= (1 << 31), b - (1 << 32), b).to(torch.int32)


def _popcount_dist(q, codes):
    """Hamming distance through numpy's byte unpacking (a different route from the oracle's loop)."""
    x = (codes.numpy().view(np.uint32) ^ q.numpy().view(np.uint32)[None, :])
    return np.unpackbits(x.view(np.uint8), axis=1).sum(axis=1)


# ------------------------------------------------------------------ Hamming
@pytest.mark.parametrize("W", [1, 2, 4, 8, 16])
def test_hamming_matches_unpackbits(W):
    codes = _rand_codes(W, 500, W)
    q = _rand_codes(100 + W, 1, W)[0].contiguous()
    d = oracle.hamming(q, codes).numpy()
    assert np.array_equal(d, _popcount_dist(q, codes))


def test_hamming_invariants_and_nxor_score():
    W, L = 4, 128
    codes = _rand_codes(3, 64, W)
    a, b, c = codes[0].contiguous(), codes[1].contiguous(), codes[2].contiguous()
    dist = lambda x, y: int(oracle.hamming(x, y.view(1, W))[0])
    assert dist(a, a) == 0
    assert dist(a, (~a).contiguous()) == L
    assert dist(a, b) == dist(b, a)
    assert dist(a, c) <= dist(a, b) + dist(b, c)
    # flipping exactly one bit moves the distance by exactly one
    flipped = a.clone()
    flipped[2] ^= (1 << 7)
    assert dist(a, flipped) == 1
    # sign bit of a word counts like any other
    flipped = a.clone()
    flipped[1] ^= -(1 << 31)
    assert dist(a, flipped) == 1
    # Eq. 3's NXOR/popcount score is the number of agreeing bits
    for y in (a, b, c):
        assert oracle.nxor_score(a, y) == L - dist(a, y)


def test_hamming_does_not_depend_on_bit_layout():
    """Distances between hashed vectors equal the count of differing sign bits before packing."""
    cfg = wl.CONFIGS["C1"].scaled(n_tokens=64, needles=0)
    w = wl.Workload(cfg)
    w1, b1, w2 = w.hash_weights()
    K = w.kv_rows("K", 0, 0, 0, 64)
    bits, codes = oracle.hash_rows(K, w1[0], b1[0], w2[0], cfg.code_bits)
    qbits, qcode = oracle.hash_rows(w.q[0], w1[0], b1[0], w2[0], cfg.code_bits)
    want = (bits != qbits).sum(dim=1).to(torch.int16)
    assert torch.equal(oracle.hamming(qcode[0].contiguous(), codes), want)


# ------------------------------------------------------------------ top-k
def test_topk_matches_stable_sort():
    rng = np.random.default_rng(5)
    for n, k in [(1, 1), (10, 3), (1000, 20), (1000, 1000), (4096, 128)]:
        dist = torch.from_numpy(rng.integers(40, 90, size=n).astype(np.int16))
        order = np.argsort(dist.numpy(), kind="stable")[:k]      # ties keep the lower index first
        want = np.sort(order).astype(np.int32)
        assert np.array_equal(oracle.topk(dist, k).numpy(), want), (n, k)


def test_topk_brute_force_tiny():
    """Every size-k subset is tried; the winner minimises (sum of distances, then indices)."""
    import itertools
    rng = np.random.default_rng(6)
    for _ in range(20):
        n, k = 7, 3
        dist = rng.integers(0, 4, size=n)
        best = min(itertools.combinations(range(n), k),
                   key=lambda s: (sorted(dist[list(s)].tolist(), reverse=True), s))
        # the set minimising the sorted-descending distance vector lexicographically, ties by index
        got = oracle.topk(torch.from_numpy(dist.astype(np.int16)), k).tolist()
        assert got == list(best), (dist, got, best)


def test_topk_special_cases():
    n = 257
    assert oracle.topk(torch.zeros(n, dtype=torch.int16), 9).tolist() == list(range(9))
    d = torch.full((n,), 60, dtype=torch.int16)
    d[200] = 3
    d[17] = 3
    assert oracle.topk(d, 1).tolist() == [17]             # lowest index among the minima
    assert oracle.topk(d, 2).tolist() == [17, 200]
    assert oracle.topk(d, 4).tolist() == [0, 1, 17, 200]  # ties filled from the low end, output ascending
    assert oracle.topk(d, n).tolist() == list(range(n))
    with pytest.raises(ValueError):
        oracle.topk(d, n + 1)
    with pytest.raises(ValueError):
        oracle.topk(d, 0)


# ------------------------------------------------------------------ attention
def _dense_softmax_attention(q, K, V, scale):
    s = (K.double().numpy() @ q.double().numpy()) * scale
    p = np.exp(s - s.max())
    p /= p.sum()
    return p @ V.double().numpy()


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_attention_k_equals_n_is_full_attention(dtype):
    """With I = all cached tokens, the gathered attention is Eq. 1 over the cache."""
    n, d = 300, 128
    q = wl.normal(1, 1, 0, d).to(dtype)
    K = wl.normal(1, 2, 0, n * d).view(n, d).to(dtype).contiguous()
    V = wl.normal(1, 3, 0, n * d).view(n, d).to(dtype).contiguous()
    scale = 1.0 / math.sqrt(d)
    out = oracle.sparse_attention(q, K, V, torch.arange(n, dtype=torch.int32), scale).numpy()
    want = _dense_softmax_attention(q, K, V, scale)
    assert np.max(np.abs(out - want)) < 1e-6


def test_attention_restricted_to_subset_and_order_free():
    n, d, k = 500, 128, 37
    q = wl.normal(2, 1, 0, d)
    K = wl.normal(2, 2, 0, n * d).view(n, d).contiguous()
    V = wl.normal(2, 3, 0, n * d).view(n, d).contiguous()
    idx = torch.from_numpy(np.sort(np.random.default_rng(0).choice(n, k, replace=False)).astype(np.int32))
    scale = 0.31
    out = oracle.sparse_attention(q, K, V, idx, scale).numpy()
    sel = idx.long()
    want = _dense_softmax_attention(q, K[sel], V[sel], scale)
    assert np.max(np.abs(out - want)) < 1e-6
    perm = idx[torch.from_numpy(np.random.default_rng(1).permutation(k))].contiguous()
    out2 = oracle.sparse_attention(q, K, V, perm, scale).numpy()
    assert np.max(np.abs(out - out2)) < 1e-6
    # scale matters: a different scale gives a different answer
    out3 = oracle.sparse_attention(q, K, V, idx, 2 * scale).numpy()
    assert np.max(np.abs(out - out3)) > 1e-3


def test_attention_closed_forms():
    n, d = 64, 128
    q = wl.normal(3, 1, 0, d)
    K = wl.normal(3, 2, 0, n * d).view(n, d).contiguous()
    V = wl.normal(3, 3, 0, n * d).view(n, d).contiguous()
    # one row: softmax over a single score is 1
    out = oracle.sparse_attention(q, K, V, torch.tensor([41], dtype=torch.int32), 0.1)
    assert torch.equal(out, V[41])
    # equal keys: uniform weights, the output is the mean of the gathered values
    Keq = K[:1].repeat(n, 1).contiguous()
    idx = torch.tensor([3, 9, 10, 50], dtype=torch.int32)
    out = oracle.sparse_attention(q, Keq, V, idx, 0.1).numpy()
    assert np.allclose(out, V[idx.long()].double().mean(0).numpy(), atol=1e-6)
    # a key far along q takes all the weight
    Kn = K.clone()
    Kn[20] = 50 * q
    out = oracle.sparse_attention(q, Kn, V, torch.arange(n, dtype=torch.int32), 1.0).numpy()
    assert np.allclose(out, V[20].numpy(), atol=1e-5)


# ------------------------------------------------------------------ the layer-level chain
def test_layer_chain_on_config_c1_finds_planted_needles():
    cfg = wl.CONFIGS["C1"]
    w = wl.Workload(cfg)
    w1, b1, w2 = w.hash_weights()
    K = w.materialize("K", "cpu")
    V = w.materialize("V", "cpu")
    codes = torch.zeros(cfg.batch, cfg.n_kv_heads, cfg.max_tokens, cfg.words, dtype=torch.int32)
    oracle.hash_keys(K, w1, b1, w2, cfg.code_bits, 0, cfg.n_tokens, codes)
    idx, qcode, dist = oracle.retrieve_topk(w.q, w1, b1, w2, codes, cfg.n_tokens, cfg.topk, want_dist=True)
    # composition of the single steps
    _, qc = oracle.hash_rows(w.q[0], w1[0], b1[0], w2[0], cfg.code_bits)
    assert torch.equal(qcode[0], qc)
    dd = oracle.hamming(qc[0].contiguous(), codes[0, 0, :cfg.n_tokens].contiguous())
    assert torch.equal(dist[0, 0], dd)
    assert torch.equal(idx[0, 0], oracle.topk(dd, cfg.topk))
    # needles are copies of q: distance 0, so all of them are selected
    needles = set(w.needle_pos[0, 0].tolist())
    assert len(needles) == cfg.needles
    assert all(int(dist[0, 0, p]) == 0 for p in needles)
    assert needles <= set(idx[0, 0].tolist())
    # selected distances never exceed unselected ones
    mask = torch.zeros(cfg.n_tokens, dtype=torch.bool)
    mask[idx[0, 0].long()] = True
    assert int(dist[0, 0][mask].max()) <= int(dist[0, 0][~mask].min())
    # attention: with needles (logit |q|^2/sqrt(d) far above the rest) the output is close to the
    # needles' mean value row
    out = oracle.sparse_decode(w.q, K, V, idx, 1.0 / math.sqrt(cfg.head_dim))
    sel = idx[0, 0].long()
    want = _dense_softmax_attention(w.q[0, 0], K[0, 0][sel], V[0, 0][sel], 1.0 / math.sqrt(cfg.head_dim))
    assert np.max(np.abs(out[0, 0].numpy() - want)) < 1e-6
    # k = N reproduces full attention over the cache
    full = torch.arange(cfg.n_tokens, dtype=torch.int32).view(1, 1, -1).contiguous()
    out_full = oracle.sparse_decode(w.q, K, V, full, 1.0 / math.sqrt(cfg.head_dim))
    want_full = _dense_softmax_attention(w.q[0, 0], K[0, 0, :cfg.n_tokens], V[0, 0, :cfg.n_tokens],
                                         1.0 / math.sqrt(cfg.head_dim))
    assert np.max(np.abs(out_full[0, 0].numpy() - want_full)) < 1e-6


def test_gqa_head_mapping():
    """Query head hq reads kv head hq // group: codes, weights, K and V."""
    cfg = wl.CONFIGS["C4"].scaled(batch=2, n_q_heads=4, n_kv_heads=2, n_tokens=200, topk=10,
                                  hidden=64, code_bits=64, needles=2)
    w = wl.Workload(cfg)
    w1, b1, w2 = w.hash_weights()
    K = w.materialize("K", "cpu")
    V = w.materialize("V", "cpu")
    codes = torch.zeros(cfg.batch, cfg.n_kv_heads, cfg.max_tokens, cfg.words, dtype=torch.int32)
    oracle.hash_keys(K, w1, b1, w2, cfg.code_bits, 0, cfg.n_tokens, codes)
    idx, qcode, dist = oracle.retrieve_topk(w.q, w1, b1, w2, codes, cfg.n_tokens, cfg.topk, want_dist=True)
    out = oracle.sparse_decode(w.q, K, V, idx, 0.2)
    for b in range(cfg.batch):
        for hq in range(cfg.n_q_heads):
            hk = hq // cfg.group
            _, qc = oracle.hash_rows(w.q[b, hq:hq + 1].contiguous(), w1[hk], b1[hk], w2[hk], cfg.code_bits)
            assert torch.equal(qcode[b, hq], qc[0])
            dd = oracle.hamming(qc[0].contiguous(), codes[b, hk, :cfg.n_tokens].contiguous())
            assert torch.equal(dist[b, hq], dd)
            assert set(w.needle_pos[b, hq].tolist()) <= set(idx[b, hq].tolist())
            o = oracle.sparse_attention(w.q[b, hq].contiguous(), K[b, hk], V[b, hk], idx[b, hq].contiguous(), 0.2)
            assert torch.equal(out[b, hq], o)
