"""Pins for the oracle's hashing and bit-packing (CPU only).

The oracle is checked against things that are not the oracle: the paper's packing rule worked by
hand (tests/golden/bit_packing.txt), closed forms of special MLPs, libm's exp, and an fp64
evaluation built from numpy matmuls.
"""
import math
import os

import numpy as np
import pytest
import torch

import oracle
import workload as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _u32(t):
    return t.numpy().astype(np.int64) & 0xFFFFFFFF


def _golden_packing():
    rows = []
    for line in open(os.path.join(GOLDEN, "bit_packing.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        L, ones, words = [s.strip() for s in line.split(";")]
        rows.append((int(L), [int(x) for x in ones.split()], [int(x, 16) for x in words.split()]))
    return rows


@pytest.mark.parametrize("L,ones,words", _golden_packing())
def test_pack_hand_worked(L, ones, words):
    bits = torch.zeros(1, L, dtype=torch.uint8)
    bits[0, ones] = 1
    got = _u32(oracle.pack_bits(bits))[0].tolist()
    assert got == words


@pytest.mark.parametrize("L", [32, 64, 96, 128, 256, 512])
def test_pack_matches_chunk_shift_or(L):
    """The appendix's procedure carried out with numpy array ops on a random boolean matrix."""
    rng = np.random.default_rng(L)
    bits = rng.integers(0, 2, size=(37, L), dtype=np.uint8)
    out = np.zeros((37, L // 32), dtype=np.uint64)
    for chunk in np.split(bits, 32, axis=-1):
        out = (out << np.uint64(1)) | chunk.astype(np.uint64)
    got = _u32(oracle.pack_bits(torch.from_numpy(bits)))
    assert np.array_equal(got, out.astype(np.int64))
    # every bit is used exactly once: unpacking by the index rule restores the matrix
    W = L // 32
    back = np.zeros_like(bits)
    for c in range(32):
        for j in range(W):
            back[:, c * W + j] = (got[:, j] >> (31 - c)) & 1
    assert np.array_equal(back, bits)


def test_exp_routine_against_libm():
    worst = 0.0
    for t in np.linspace(-87.0, 88.0, 35001):
        t32 = float(np.float32(t))
        ref = math.exp(t32)
        got = oracle.exp32(t32)
        worst = max(worst, abs(got - ref) / ref)
    assert worst < 2.5e-7, worst          # about two units in the last place of binary32
    assert oracle.exp32(0.0) == 1.0
    # clamped ends, and NaN treated as the lower end
    assert oracle.exp32(-1000.0) == oracle.exp32(-87.0)
    assert oracle.exp32(1000.0) == oracle.exp32(88.0)
    assert oracle.exp32(float("nan")) == oracle.exp32(-87.0)


def test_silu_against_definition():
    for a in np.linspace(-30, 30, 6001):
        a32 = float(np.float32(a))
        ref = a32 / (1.0 + math.exp(-a32))
        got = oracle.silu32(a32)
        assert abs(got - ref) <= 4e-7 * max(abs(ref), 1e-30) + 1e-37, (a32, got, ref)
    assert oracle.silu32(0.0) == 0.0
    assert oracle.silu32(200.0) == 200.0
    assert abs(oracle.silu32(-200.0)) < 1e-30


def test_identity_mlp_gives_sign_of_input():
    """W1 = I, b1 = 0, W2 = I: y_j = SiLU(x_j), whose sign is the sign of x_j; zeros give bit 0."""
    d = 128
    x = wl.normal(11, 1, 0, 50 * d).view(50, d).contiguous()
    x[0, :5] = 0.0
    x[1, 7] = -0.0
    eye = torch.eye(d)
    bits, codes = oracle.hash_rows(x, eye, torch.zeros(d), eye, d)
    assert torch.equal(bits, (x > 0).to(torch.uint8))
    assert torch.equal(codes, oracle.pack_bits(bits))


def test_linear_hash_with_identity_rotation():
    """hidden = 0 is Eq. 4, sign(xR); with R = I the code is the sign pattern of x itself."""
    d = 128
    x = wl.normal(12, 1, 0, 20 * d).view(20, d).to(torch.bfloat16).contiguous()
    bits, _ = oracle.hash_rows(x, torch.eye(d).to(torch.bfloat16), None, None, d)
    assert torch.equal(bits, (x.float() > 0).to(torch.uint8))


def test_linear_hash_is_row_times_R_not_transposed():
    """A non-symmetric R tells W[j][k] (row = hash output) from its transpose."""
    d, L = 128, 32
    R = torch.zeros(L, d)
    R[0, 5] = 1.0       # output 0 looks at x[5]
    R[3, 0] = -1.0      # output 3 looks at -x[0]
    x = torch.zeros(1, d)
    x[0, 5] = 2.0
    x[0, 0] = -3.0
    bits, _ = oracle.hash_rows(x, R, None, None, L)
    want = torch.zeros(1, L, dtype=torch.uint8)
    want[0, 0] = 1
    want[0, 3] = 1
    assert torch.equal(bits, want)


def test_bias_and_second_layer_are_used():
    """One hidden unit driven only by its bias: y_j = W2[j][0]*SiLU(b1_0)."""
    d, h, L = 128, 4, 32
    w1 = torch.zeros(h, d)
    b1 = torch.tensor([2.0, 0.0, 0.0, 0.0])
    w2 = torch.zeros(L, h)
    w2[:, 0] = torch.tensor([1.0 if j % 3 == 0 else -1.0 for j in range(L)])
    x = wl.normal(5, 1, 0, d).view(1, d).contiguous()
    bits, _, y = oracle.hash_rows(x, w1, b1, w2, L, want_y=True)
    assert bits[0].tolist() == [1 if j % 3 == 0 else 0 for j in range(L)]
    silu2 = 2.0 / (1.0 + math.exp(-2.0))
    assert np.allclose(y[0].numpy(), w2[:, 0].numpy() * silu2, rtol=1e-6)
    # negative pre-activation gives a negative SiLU: the signs flip
    bits_neg, _ = oracle.hash_rows(x, w1, -b1, w2, L)
    assert bits_neg[0].tolist() == [0 if j % 3 == 0 else 1 for j in range(L)]


@pytest.mark.parametrize("wdt,xdt", [(torch.float32, torch.float32), (torch.bfloat16, torch.bfloat16)])
def test_mlp_signs_agree_with_fp64_where_margin_is_clear(wdt, xdt):
    """The binary32 chain and an fp64 evaluation (numpy matmul + numpy exp, and the oracle's own
    fp64 routine) give the same sign wherever |y| is well above binary32 round-off."""
    cfg = wl.CONFIGS["C2"].scaled(n_kv_heads=2, n_q_heads=2, n_tokens=256, needles=0,
                                  kv_dtype="f32" if xdt == torch.float32 else "bf16",
                                  weight_dtype="f32" if wdt == torch.float32 else "bf16")
    w = wl.Workload(cfg)
    w1, b1, w2 = w.hash_weights()
    x = w.kv_rows("K", 0, 1, 0, 256)
    bits, codes, y32 = oracle.hash_rows(x, w1[1], b1[1], w2[1], cfg.code_bits, want_y=True)
    # numpy: library matmul + exp
    xd, w1d, b1d, w2d = (t.double().numpy() for t in (x, w1[1], b1[1], w2[1]))
    a = xd @ w1d.T + b1d
    hcol = a / (1.0 + np.exp(-a))
    y_np = hcol @ w2d.T
    mag = np.abs(hcol) @ np.abs(w2d).T
    y64, mag64 = oracle.hash_margin_f64(x, w1[1], b1[1], w2[1], cfg.code_bits)
    assert np.allclose(y64.numpy(), y_np, rtol=1e-10, atol=1e-12)
    assert np.allclose(mag64.numpy(), mag, rtol=1e-10)
    clear = np.abs(y_np) > 1e-4 * mag
    assert clear.mean() > 0.99
    assert np.array_equal(bits.numpy()[clear], (y_np > 0)[clear].astype(np.uint8))
    # and the binary32 outputs are close to the fp64 ones in absolute terms
    assert np.max(np.abs(y32.numpy() - y_np) / mag) < 2e-6
    # codes are the packed bits
    assert torch.equal(codes, oracle.pack_bits(bits))
    # roughly balanced bits with seeded Gaussian weights (sanity of the workload, not a pin)
    assert 0.2 < bits.float().mean() < 0.8


def test_hash_keys_layout_and_append():
    """Layer-level call writes rows [t0, t0+n) of the right (b, head) slab and nothing else."""
    cfg = wl.CONFIGS["C2"].scaled(batch=2, n_kv_heads=2, n_q_heads=4, n_tokens=24, extra_tokens=8,
                                  needles=0)
    w = wl.Workload(cfg)
    w1, b1, w2 = w.hash_weights()
    K = w.materialize("K", "cpu")
    codes = torch.full((2, 2, cfg.max_tokens, cfg.words), 0x5A5A5A5A, dtype=torch.int32)
    oracle.hash_keys(K, w1, b1, w2, cfg.code_bits, 3, 10, codes)
    for b in range(2):
        for h in range(2):
            _, want = oracle.hash_rows(K[b, h, 3:13].contiguous(), w1[h], b1[h], w2[h], cfg.code_bits)
            assert torch.equal(codes[b, h, 3:13], want)
            assert (codes[b, h, :3] == 0x5A5A5A5A).all() and (codes[b, h, 13:] == 0x5A5A5A5A).all()
    # different heads use different weights
    assert not torch.equal(codes[0, 0, 3:13], oracle.hash_rows(K[0, 0, 3:13].contiguous(),
                                                              w1[1], b1[1], w2[1], cfg.code_bits)[1])
