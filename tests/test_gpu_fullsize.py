"""GPU parity at the full sizes of the five workloads, in the launch configuration bench.py times.

The oracle cannot hash every key of the large configs in test time, so:
  * key codes are checked bit-exactly on whole sampled heads (C2: all heads; C5: one whole head of
    a million keys per code length, and sampled rows of three more);
  * the bulk hash's matrix-core path is compared with its all-binary32 path over the WHOLE code
    tensor (both on the device), and audited output by output inside the kernel;
  * retrieval is checked bit-exactly on EVERY head from seeded synthetic code caches (both sides
    read the same generated codes), and on the sampled heads from real hashed codes;
  * attention is checked on every head against the oracle run on the gathered rows;
  * on the remaining heads of the real chain, properties that hold at any size are checked
    (k distinct ascending in-range indices, planted needles present).
Inputs come from the seeded generator only; nothing computed by the HIP path feeds the oracle.
"""
import math
import sys

import pytest
import torch

import oracle
import workload as wl
from gpu_common import torch_dtype

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]
ATTN_TOL = 2e-3
DEV = "cuda:0"


def progress(msg):
    """A line on the real stderr, flushed: the million-token tests run for minutes."""
    sys.__stderr__.write(f"  [{msg}]\n")
    sys.__stderr__.flush()


class Big:
    """Device tensors of a full-size config; host copies only of what a check needs."""

    def __init__(self, cfg, need_kv=True):
        import paper_2508_19740_amd as sp
        self.cfg = cfg
        self.w = wl.Workload(cfg)
        self.K = self.w.materialize("K", DEV) if need_kv else None
        self.V = self.w.materialize("V", DEV) if need_kv else None
        self.q = self.w.q.to(DEV)
        self.hweights = self.w.hash_weights()
        self.weights = tuple(None if t is None else t.to(DEV) for t in self.hweights)
        self.codes = torch.zeros(cfg.batch, cfg.n_kv_heads, cfg.max_tokens, cfg.words, dtype=torch.int32, device=DEV)
        self.ctx = sp.Spotlight(cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.code_bits, cfg.hidden,
                                cfg.max_tokens, cfg.topk, kv_dtype=torch_dtype(cfg.kv_dtype),
                                weight_dtype=torch_dtype(cfg.weight_dtype), device=DEV)
        self.scale = 1.0 / math.sqrt(cfg.head_dim)

    def head_weights(self, hk):
        return tuple(None if t is None else t[hk].contiguous() for t in self.hweights)

    def synthetic_codes(self):
        c = self.cfg
        out = torch.empty_like(self.codes)
        for b in range(c.batch):
            for hk in range(c.n_kv_heads):
                out[b, hk] = self.w.synthetic_codes(b, hk, 0, c.max_tokens, DEV)
        return out

    def close(self):
        self.ctx.close()


def check_index_properties(idx, cfg, needle_pos=None):
    """k distinct, ascending, in-range indices per head (and the planted needles among them)."""
    i64 = idx.long()
    assert int(i64.min()) >= 0 and int(i64.max()) < cfg.n_tokens
    assert bool((i64[..., 1:] > i64[..., :-1]).all())
    if needle_pos is not None and needle_pos.numel():
        for b in range(cfg.batch):
            for hq in range(cfg.n_q_heads):
                have = set(idx[b, hq].tolist())
                assert set(needle_pos[b, hq].tolist()) <= have, (b, hq)


def check_retrieval_on_synthetic_codes(big, n_tokens=None):
    """Every head: GPU top-k from generated codes against the oracle's full sort of the same codes."""
    c = big.cfg
    n = c.n_tokens if n_tokens is None else n_tokens
    dcodes = big.synthetic_codes()
    qcode = torch.empty(c.batch, c.n_q_heads, c.words, dtype=torch.int32, device=DEV)
    idx = big.ctx.retrieve_topk(big.q, *big.weights, dcodes, n, c.topk, out_qcode=qcode).cpu()
    qc = qcode.cpu()
    G = c.group
    for b in range(c.batch):
        for hk in range(c.n_kv_heads):
            hc = dcodes[b, hk, :n].cpu().contiguous()
            for g in range(G):
                hq = hk * G + g
                # the query code itself is pinned against the oracle's hash of q
                _, want_q = oracle.hash_rows(big.w.q[b, hq:hq + 1].contiguous(), *big.head_weights(hk), c.code_bits)
                assert torch.equal(qc[b, hq], want_q[0]), (b, hq)
                dist = oracle.hamming(want_q[0].contiguous(), hc)
                want = oracle.topk(dist, c.topk)
                assert torch.equal(idx[b, hq], want), (b, hq)
    return idx


def check_decode_step_on_synthetic_codes(big, n_sink=4, n_local=64, attn_every=1, k=None):
    """Every head: the one-call step (appended key hashed into generated codes, forced sink / local
    tokens, attention) against the oracle's single steps on the same codes (attention on every
    attn_every-th head)."""
    c = big.cfg
    n = c.n_tokens
    G = c.group
    k = c.topk if k is None else k
    dcodes = big.synthetic_codes()
    idx, out = big.ctx.decode_step(big.q, big.K, big.V, *big.weights, dcodes, n, k, n_sink, n_local)
    idx, out = idx.cpu(), out.cpu()
    ar = torch.arange(k, dtype=torch.int32)
    worst = 0.0
    for b in range(c.batch):
        for hk in range(c.n_kv_heads):
            hc = big.w.synthetic_codes(b, hk, 0, n, "cpu").contiguous()
            # the appended key's code, by the oracle from the generator's K row
            krow = big.w.kv_rows("K", b, hk, n - 1, 1, "cpu")
            _, new_code = oracle.hash_rows(krow.contiguous(), *big.head_weights(hk), c.code_bits)
            hc[n - 1] = new_code[0]
            assert torch.equal(dcodes[b, hk, n - 1].cpu(), new_code[0]), (b, hk)
            for g in range(G):
                hq = hk * G + g
                _, qc = oracle.hash_rows(big.w.q[b, hq:hq + 1].contiguous(), *big.head_weights(hk), c.code_bits)
                dist = oracle.hamming(qc[0].contiguous(), hc)
                want = oracle.topk_forced(dist, k, n_sink, n_local)
                assert torch.equal(idx[b, hq], want), (b, hq)
                if (b * c.n_q_heads + hq) % attn_every:
                    continue
                sel = want.long().to(DEV)
                Ks = big.K[b, hk].index_select(0, sel).cpu()
                Vs = big.V[b, hk].index_select(0, sel).cpu()
                o = oracle.sparse_attention(big.w.q[b, hq].contiguous(), Ks, Vs, ar, big.scale)
                worst = max(worst, float((out[b, hq] - o).abs().max()))
    assert worst <= ATTN_TOL, worst


def check_attention_all_heads(big, idx_host):
    """Every head: GPU attention over idx against the oracle on the gathered rows."""
    c = big.cfg
    didx = idx_host.to(DEV)
    out = big.ctx.sparse_decode(big.q, big.K, big.V, didx, big.scale).cpu()
    G = c.group
    ar = torch.arange(c.topk, dtype=torch.int32)
    worst = 0.0
    for b in range(c.batch):
        for hq in range(c.n_q_heads):
            sel = didx[b, hq].long()
            Ks = big.K[b, hq // G].index_select(0, sel).cpu()
            Vs = big.V[b, hq // G].index_select(0, sel).cpu()
            want = oracle.sparse_attention(big.w.q[b, hq].contiguous(), Ks, Vs, ar, big.scale)
            worst = max(worst, float((out[b, hq] - want).abs().max()))
    assert worst <= ATTN_TOL, worst


def check_bulk_hash_paths_agree(big, n_rows=None):
    """The whole code tensor, twice: second hash layer on the matrix cores (certified signs, the
    rest recomputed) and everything on the binary32 chain.  Both on the device, every word compared.
    Then the matrix-core call again with the audit on: the kernel evaluates every output with the
    chain as well and reports how far the matrix cores were from it, in units of the bound's scale."""
    import paper_2508_19740_amd as sp
    c = big.cfg
    n = c.n_tokens if n_rows is None else n_rows
    big.codes.zero_()
    big.ctx.hash_keys(big.K, *big.weights, 0, n, big.codes)
    other = torch.zeros_like(big.codes)
    big.ctx.set_option(sp.OPT_BULK_HASH_MATRIX_CORES, 0)
    try:
        big.ctx.hash_keys(big.K, *big.weights, 0, n, other)
    finally:
        big.ctx.set_option(sp.OPT_BULK_HASH_MATRIX_CORES, 1)
    assert torch.equal(big.codes, other)
    other.zero_()
    big.ctx.set_option(sp.OPT_BULK_HASH_AUDIT, 1)
    try:
        big.ctx.hash_keys(big.K, *big.weights, 0, n, other)
    finally:
        big.ctx.set_option(sp.OPT_BULK_HASH_AUDIT, 0)
    au = big.ctx.bulk_hash_audit_read()
    assert torch.equal(big.codes, other)
    del other
    progress(f"[bulk hash audit] {c.name}: outputs {au['outputs']}, recomputed {au['listed']} "
          f"({au['listed'] / au['outputs']:.3e}), largest |y_mfma - y_chain| / (|W2[j]| |h|) = {au['max_ratio']:.3e} "
          f"against eps = {au['eps']:.3e} (slack x{au['eps'] / max(au['max_ratio'], 1e-30):.1f})")
    assert au["outputs"] == c.batch * c.n_kv_heads * n * c.code_bits      # the matrix-core path did run
    assert au["wrong"] == 0
    assert au["max_ratio"] < au["eps"]
    assert au["listed"] < au["outputs"] // 100


def check_sampled_heads_real_chain(big, heads, distances=False, rehash=True):
    """Whole heads through hash -> retrieve -> attend on both sides; the GPU ran every head.
    With distances=True every distance of the sampled heads is compared as well."""
    c = big.cfg
    G = c.group
    if rehash:
        big.codes.zero_()
        big.ctx.hash_keys(big.K, *big.weights, 0, c.n_tokens, big.codes)
    dist_dev = None
    if distances:
        dist_dev = torch.empty(c.batch, c.n_q_heads, c.n_tokens, dtype=torch.int16, device=DEV)
    idx = big.ctx.retrieve_topk(big.q, *big.weights, big.codes, c.n_tokens, c.topk, out_dist=dist_dev)
    out = big.ctx.sparse_decode(big.q, big.K, big.V, idx, big.scale).cpu()
    idx_h = idx.cpu()
    check_index_properties(idx_h, c, big.w.needle_pos)
    for (b, hk) in heads:
        hK = big.K[b, hk, :c.n_tokens].cpu()
        hV = big.V[b, hk, :c.n_tokens].cpu()
        _, want_codes = oracle.hash_rows(hK, *big.head_weights(hk), c.code_bits)
        assert torch.equal(big.codes[b, hk, :c.n_tokens].cpu(), want_codes), (b, hk)
        for g in range(G):
            hq = hk * G + g
            _, qc = oracle.hash_rows(big.w.q[b, hq:hq + 1].contiguous(), *big.head_weights(hk), c.code_bits)
            dist = oracle.hamming(qc[0].contiguous(), want_codes)
            if distances:
                assert torch.equal(dist_dev[b, hq].cpu(), dist), (b, hq)
            want_idx = oracle.topk(dist, c.topk)
            assert torch.equal(idx_h[b, hq], want_idx), (b, hq)
            want = oracle.sparse_attention(big.w.q[b, hq].contiguous(), hK, hV, want_idx, big.scale)
            assert float((out[b, hq] - want).abs().max()) <= ATTN_TOL, (b, hq)
    return idx_h


def test_c2_every_head_against_the_full_oracle():
    big = Big(wl.CONFIGS["C2"])
    try:
        c = big.cfg
        idx = check_sampled_heads_real_chain(big, [(0, h) for h in range(c.n_kv_heads)])
        check_attention_all_heads(big, idx)
        # the one-call step as the five launches of the general path, and as ONE kernel launch (an
        # option; that it is what ran is checked)
        import paper_2508_19740_amd as sp
        big.ctx.prepack_weights(*big.weights)
        check_decode_step_on_synthetic_codes(big)
        big.ctx.set_option(sp.OPT_STEP_SINGLE_LAUNCH, 1)
        big.ctx.profile_enable(True)
        check_decode_step_on_synthetic_codes(big)
        ran = big.ctx.profile_read()
        big.ctx.profile_enable(False)
        assert ran["step_small"][1] == 1 and ran["score"][1] == 0
    finally:
        big.close()


def test_c3_512k_tokens():
    big = Big(wl.CONFIGS["C3"])
    try:
        check_bulk_hash_paths_agree(big)
        idx = check_sampled_heads_real_chain(big, [(0, 5), (0, 31)], distances=True, rehash=False)
        check_attention_all_heads(big, idx)
        check_retrieval_on_synthetic_codes(big)
        big.ctx.prepack_weights(*big.weights)      # as bench.py runs the step
        check_decode_step_on_synthetic_codes(big)
    finally:
        big.close()


def test_c4_gqa_batch16():
    big = Big(wl.CONFIGS["C4"])
    try:
        check_bulk_hash_paths_agree(big)
        idx = check_sampled_heads_real_chain(big, [(0, 0), (9, 3), (15, 7)], rehash=False)
        check_attention_all_heads(big, idx)
        check_retrieval_on_synthetic_codes(big)
        big.ctx.prepack_weights(*big.weights)      # as bench.py runs the step
        check_decode_step_on_synthetic_codes(big, attn_every=7)
    finally:
        big.close()


def test_groups_of_seven_at_128k_tokens():
    """Qwen2.5-7B's attention layout (28 query heads on 4 key-value heads) at a 128K context: every
    head through the whole chain on both sides."""
    big = Big(wl.CONFIGS["Q7-128K"])
    try:
        c = big.cfg
        idx = check_sampled_heads_real_chain(big, [(0, h) for h in range(c.n_kv_heads)], distances=True)
        check_attention_all_heads(big, idx)
        big.ctx.prepack_weights(*big.weights)
        check_decode_step_on_synthetic_codes(big)
    finally:
        big.close()


@pytest.mark.parametrize("words", [2, 5])
def test_many_blocks_of_many_heads(words):
    """512 query heads x 9 token blocks: more (head, block) pairs than the chip holds at once, which
    is where retrieval switches to its single-wavefront select kernel; with and without forced
    tokens, for code lengths other than those of C4 and C5."""
    cfg = wl.CONFIGS["C4"].scaled(batch=8, n_q_heads=64, n_kv_heads=8, n_tokens=8 * 4096 + 77, topk=9400,
                                  hidden=128, code_bits=32 * words, needles=0, seed=4242 + words)
    big = Big(cfg)
    try:
        check_decode_step_on_synthetic_codes(big, n_sink=0, n_local=0, attn_every=61, k=300)
        check_decode_step_on_synthetic_codes(big, n_sink=4, n_local=64, attn_every=67, k=300)
        big.ctx.prepack_weights(*big.weights)
        check_decode_step_on_synthetic_codes(big, n_sink=5000, n_local=4100, attn_every=509, k=9400)   # windows wider than a block
    finally:
        big.close()


@pytest.mark.parametrize("shape", [(1, 32, 32, 40 * 4096 + 100, 4), (2, 32, 16, 69 * 4096 + 4000, 3), (1, 8, 1, 700 * 4096 + 9, 8),
                                   (1, 4, 4, 599 * 4096 + 77, 4), (1, 8, 8, 601 * 4096 + 5, 2)])
def test_runs_of_blocks_that_straddle_heads(shape):
    """More (kv head, block) tasks than resident score workgroups, so that a workgroup counts a run
    of two or three consecutive blocks, with block counts that are no multiple of the run length
    (runs then start in one head and end in the next); one head of 701 blocks on its own; and heads
    with more runs than a select workgroup has threads (200 runs of 3 blocks with 128 threads, 121
    runs of 5 with 64).  The select kernel rebuilds every block's counts and offsets from the runs'
    cumulative histograms."""
    batch, hq, hkv, n, words = shape
    k = max(2000, n // 300)
    cfg = wl.CONFIGS["C3"].scaled(batch=batch, n_q_heads=hq, n_kv_heads=hkv, n_tokens=n, topk=k + 4300,
                                  hidden=128, code_bits=32 * words, needles=0, seed=777 + hq + words)
    big = Big(cfg)
    try:
        check_decode_step_on_synthetic_codes(big, n_sink=0, n_local=0, attn_every=13, k=k)
        check_decode_step_on_synthetic_codes(big, n_sink=4, n_local=4200, attn_every=17, k=k + 4300)
    finally:
        big.close()


@pytest.fixture(scope="module")
def c5_kv():
    """K and V of config C5 (the 128-bit and 512-bit variants share them): 2 x 34 GB on the device."""
    w = wl.Workload(wl.CONFIGS["C5-128"])
    return w.materialize("K", DEV), w.materialize("V", DEV)


C5_WHOLE_HEAD = {"C5-128": (2, 17), "C5-512": (1, 9)}


@pytest.mark.parametrize("name", ["C5-128", "C5-512"])
def test_c5_one_million_tokens_with_growth(c5_kv, name):
    """Config C5 as the other configs are checked, plus its cache growth: one whole (batch, head)
    of a million keys goes hash -> retrieve -> attend on both sides; then the config's 64 decode
    steps run through spotlight_decode_step, each appending one key per head; every appended code
    of every head is compared with the oracle's, and on the whole head the index arrays and the
    attention output are compared after steps 1, 32 and 64."""
    big = Big(wl.CONFIGS[name], need_kv=False)
    big.K, big.V = c5_kv
    try:
        c = big.cfg
        N, k, steps = c.n_tokens, c.topk, c.extra_tokens
        assert steps == 64
        # bulk build on the matrix cores; for the long codes (hidden 1024, four code words per
        # wavefront) also against the all-binary32 path over the whole tensor, and audited
        progress(f"{name}: bulk hash")
        if name == "C5-512":
            check_bulk_hash_paths_agree(big, n_rows=N)
        else:
            big.ctx.hash_keys(big.K, *big.weights, 0, N, big.codes)
        assert int(big.codes[:, :, N:].abs().max()) == 0              # rows never hashed stay untouched
        # sampled rows of sampled heads, including both ends and a tile boundary
        gen = torch.Generator().manual_seed(7)
        rows = torch.cat([torch.arange(0, 40), torch.arange(N // 2 - 20, N // 2 + 20), torch.arange(N - 40, N),
                          torch.randint(0, N, (400,), generator=gen)]).unique()
        for (b, hk) in [(0, 0), (2, 17), (3, 31)]:
            x = big.K[b, hk].index_select(0, rows.to(DEV)).cpu()
            _, want = oracle.hash_rows(x, *big.head_weights(hk), c.code_bits)
            got = big.codes[b, hk].index_select(0, rows.to(DEV)).cpu()
            assert torch.equal(got, want), (b, hk)
        # one whole head: all N + 64 codes by the oracle (the last 64 are the keys the steps append)
        wb, wh = C5_WHOLE_HEAD[name]
        progress(f"{name}: the oracle hashes head {(wb, wh)}")
        hK = big.K[wb, wh].cpu()
        hV = big.V[wb, wh].cpu()
        _, head_codes = oracle.hash_rows(hK, *big.head_weights(wh), c.code_bits)
        assert torch.equal(big.codes[wb, wh, :N].cpu(), head_codes[:N]), (wb, wh)
        _, qc = oracle.hash_rows(big.w.q[wb, wh:wh + 1].contiguous(), *big.head_weights(wh), c.code_bits)

        def check_whole_head(n, idx, out, what):
            dist = oracle.hamming(qc[0].contiguous(), head_codes[:n].contiguous())
            want_idx = oracle.topk(dist, k)
            assert torch.equal(idx[wb, wh].cpu(), want_idx), (what, n)
            want = oracle.sparse_attention(big.w.q[wb, wh].contiguous(), hK[:n], hV[:n], want_idx, big.scale)
            assert float((out[wb, wh].cpu() - want).abs().max()) <= ATTN_TOL, (what, n)
            return want_idx

        progress(f"{name}: retrieval and attention on that head, then {steps} steps")
        # before any growth: the three calls over the N cached tokens
        idx = big.ctx.retrieve_topk(big.q, *big.weights, big.codes, N, k)
        out = big.ctx.sparse_decode(big.q, big.K, big.V, idx, big.scale)
        check_whole_head(N, idx, out, "three calls")
        # the 64 steps: the appends and the query hash read the packed copy of the weights, as in bench.py
        big.ctx.prepack_weights(*big.weights)
        for j in range(steps):
            n = N + j + 1
            idx, out = big.ctx.decode_step(big.q, big.K, big.V, *big.weights, big.codes, n, k)
            if j + 1 in (1, 32, 64):
                check_whole_head(n, idx, out, "decode_step")
                # the same step as three calls over the same grown cache
                idx3 = big.ctx.retrieve_topk(big.q, *big.weights, big.codes, n, k)
                assert torch.equal(idx3, idx), j
        progress(f"{name}: appended codes, attention on every head, generated codes")
        # every appended code of every head
        for b in range(c.batch):
            for hk in range(c.n_kv_heads):
                x = big.K[b, hk, N:N + steps].cpu()
                _, want = oracle.hash_rows(x, *big.head_weights(hk), c.code_bits)
                assert torch.equal(big.codes[b, hk, N:N + steps].cpu(), want), (b, hk)
        # the grown cache: properties on every head, attention on every head
        idx_h = idx.cpu()
        check_index_properties(idx_h, c.scaled(n_tokens=N + steps), big.w.needle_pos)
        check_attention_all_heads(big, idx_h)
        # exact retrieval on every head from generated codes, over a ragged token count
        check_retrieval_on_synthetic_codes(big, n_tokens=N + 3)
    finally:
        big.close()
