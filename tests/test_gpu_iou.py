"""Retrieval overlap with the exact top-k of q.K^T on the synthetic cone workload, through the HIP
library: the linear LSH baseline (rotation and Gaussian initialisation, 128- and 512-bit codes)
and the untrained MLP hash.  At the small size the library's indices equal the oracle's, so the
overlaps equal those of tests/test_oracle_lsh_iou.py; at 64K tokens only the library runs.
Trained weights and the paper's data do not exist here: the numbers show the shape of the
untrained columns (longer codes retrieve better, hashing beats chance), nothing more."""
import numpy as np
import pytest
import torch

import oracle
import workload as wl
from gpu_common import Case
from test_oracle_lsh_iou import VARIANTS, BASE, exact_topk, _iou

pytestmark = pytest.mark.gpu


def _library_idx(cfg):
    c = Case(cfg, host_copy=False)
    try:
        c.ctx.hash_keys(c.K, *c.weights, 0, cfg.n_tokens, c.codes)
        idx = c.ctx.retrieve_topk(c.q, *c.weights, c.codes, cfg.n_tokens, cfg.topk)
        return idx.cpu(), c.K.cpu(), c.w.q
    finally:
        c.close()


@pytest.mark.parametrize("name", sorted(VARIANTS))
def test_small_size_equals_the_oracle(name):
    cfg = VARIANTS[name]
    idx, K, q = _library_idx(cfg)
    w = wl.Workload(cfg)
    hw = w.hash_weights()
    codes = torch.zeros(cfg.batch, cfg.n_kv_heads, cfg.max_tokens, cfg.words, dtype=torch.int32)
    oracle.hash_keys(K, *hw, cfg.code_bits, 0, cfg.n_tokens, codes)
    want, _, _ = oracle.retrieve_topk(w.q, *hw, codes, cfg.n_tokens, cfg.topk)
    assert torch.equal(idx, want)


def test_iou_at_64k_tokens():
    big = {n: c.scaled(n_tokens=65536, topk=1311, kv_dtype="bf16", weight_dtype="bf16") for n, c in VARIANTS.items()}
    iou = {}
    for name, cfg in big.items():
        idx, K, q = _library_idx(cfg)
        vals = []
        for hq in range(cfg.n_q_heads):
            s = K[0, hq].double() @ q[0, hq].double()             # exact scores of the stored values
            ex = torch.topk(s, cfg.topk).indices
            vals.append(_iou(idx[0, hq], ex))
        iou[name] = float(np.mean(vals))
    k, n = 1311, 65536
    chance = (k / n) / (2 - k / n)
    print("IoU vs exact top-k (2 % of 65536 tokens, 8 heads):", {a: round(b, 3) for a, b in iou.items()},
          "chance", round(chance, 4))
    assert iou["lsh_rot_128"] > 5 * chance
    assert iou["lsh_rot_512"] > iou["lsh_rot_128"] + 0.05
    assert iou["lsh_rot_1024"] > iou["lsh_rot_512"] + 0.03
    assert iou["lsh_gauss_128"] > 5 * chance
