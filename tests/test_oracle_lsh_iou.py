"""Linear LSH baseline (Sec. 3.2 Eq. 4, appendix "LSH Weight Initialization") and the retrieval
overlap it gives on the synthetic cone workload (CPU only, through the oracle).

The paper's Table 1 / Fig. 2a compare hash top-k against the exact top-k of q.K^T by intersection
over union on real model activations with trained weights; neither exists here.  What can be
checked without them is the shape of the untrained columns: angular LSH beats chance, and longer
codes retrieve better.  No quality claim is made for the untrained MLP hash.
"""
import math

import numpy as np
import pytest
import torch

import oracle
import workload as wl


def test_rotation_init_is_a_rotation():
    for start in (0, 128 * 128, 5 * 128 * 128):
        q = wl.rotation_matrix(0x77, wl.TAG_W1, start, 128).double()
        assert float((q.T @ q - torch.eye(128, dtype=torch.float64)).abs().max()) < 1e-6
        assert abs(float(torch.linalg.det(q)) - 1.0) < 1e-5
    a = wl.rotation_matrix(0x77, wl.TAG_W1, 0, 128)
    b = wl.rotation_matrix(0x77, wl.TAG_W1, 128 * 128, 128)
    assert not torch.equal(a, b)                                   # independent blocks
    assert torch.equal(a, wl.rotation_matrix(0x77, wl.TAG_W1, 0, 128))   # reproducible


@pytest.mark.parametrize("theta", [math.pi / 6, math.pi / 3, math.pi / 2, 2 * math.pi / 3])
def test_angular_lsh_bits_differ_with_probability_theta_over_pi(theta):
    """Closed form for sign(xR) with random hyperplanes: two vectors at angle theta disagree on a bit
    with probability theta / pi.  Eight independent rotations = 1024 hyperplanes, four vector pairs."""
    d, L = 128, 1024
    R = torch.cat([wl.rotation_matrix(0x99, wl.TAG_W1, j * d * d, d) for j in range(L // d)])   # [L, d]
    frac = []
    for pair in range(4):
        g = wl.normal(0x99, wl.TAG_Q, pair * 2 * d, 2 * d).double().view(2, d)
        x = g[0] / g[0].norm()
        p = g[1] - (g[1] @ x) * x
        p = p / p.norm()
        y = math.cos(theta) * x + math.sin(theta) * p
        bits, codes = oracle.hash_rows(torch.stack([x, y]).float().contiguous(), R.contiguous(), None, None, L)
        frac.append(float((bits[0] != bits[1]).float().mean()))
        dist = oracle.hamming(codes[0].contiguous(), codes[1:2].contiguous())
        assert int(dist[0]) == int((bits[0] != bits[1]).sum())      # packed distance = bit disagreements
    assert abs(np.mean(frac) - theta / math.pi) < 0.03, (frac, theta / math.pi)


def _iou(a: torch.Tensor, b: torch.Tensor) -> float:
    sa, sb = set(a.tolist()), set(b.tolist())
    return len(sa & sb) / len(sa | sb)


def exact_topk(q, K, n, k):
    """Indices of the k largest inner products q.K^T (the paper's "oracle top-k"), ascending."""
    s = K[:n].double() @ q.double()
    order = np.lexsort((np.arange(n), -s.numpy()))
    return torch.from_numpy(np.sort(order[:k]).astype(np.int32))


def hash_iou(cfg, n_heads=None):
    """Mean IoU over heads between the hash top-k (oracle) and the exact top-k, same k."""
    w = wl.Workload(cfg)
    hw = w.hash_weights()
    K = w.materialize("K", "cpu")
    codes = torch.zeros(cfg.batch, cfg.n_kv_heads, cfg.max_tokens, cfg.words, dtype=torch.int32)
    oracle.hash_keys(K, *hw, cfg.code_bits, 0, cfg.n_tokens, codes)
    idx, _, _ = oracle.retrieve_topk(w.q, *hw, codes, cfg.n_tokens, cfg.topk)
    vals = []
    for b in range(cfg.batch):
        for hq in range(cfg.n_q_heads):
            ex = exact_topk(w.q[b, hq].float(), K[b, hq // cfg.group].float(), cfg.n_tokens, cfg.topk)
            vals.append(_iou(idx[b, hq], ex))
    return float(np.mean(vals))


BASE = wl.CONFIGS["C2"].scaled(n_q_heads=8, n_kv_heads=8, n_tokens=4096, topk=82, needles=0, kv_dtype="f32",
                               weight_dtype="f32")
VARIANTS = {
    "lsh_rot_128": BASE.scaled(hidden=0, code_bits=128, lsh_init="rotation"),
    "lsh_rot_512": BASE.scaled(hidden=0, code_bits=512, lsh_init="rotation"),
    "lsh_rot_1024": BASE.scaled(hidden=0, code_bits=1024, lsh_init="rotation"),
    "lsh_gauss_128": BASE.scaled(hidden=0, code_bits=128),
    "mlp_untrained_128": BASE.scaled(hidden=256, code_bits=128),
}


def test_iou_shape_on_the_cone_workload():
    chance = BASE.topk / BASE.n_tokens / (2 - BASE.topk / BASE.n_tokens)   # IoU of two random k-subsets
    iou = {name: hash_iou(cfg) for name, cfg in VARIANTS.items()}
    print("IoU vs exact top-k (2 % budget, 4096 tokens, 8 heads):", {k: round(v, 3) for k, v in iou.items()},
          "chance", round(chance, 4))
    assert iou["lsh_rot_128"] > 5 * chance                   # hashing retrieves far better than chance
    assert iou["lsh_rot_512"] > iou["lsh_rot_128"] + 0.05    # longer codes retrieve better (Fig. 2a's axis)
    assert iou["lsh_rot_1024"] > iou["lsh_rot_512"] + 0.03
    assert iou["lsh_gauss_128"] > 5 * chance
    assert 0.0 <= iou["mlp_untrained_128"] <= 1.0            # untrained MLP: reported, no claim
