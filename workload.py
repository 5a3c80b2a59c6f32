"""Seeded synthetic inputs for the Spotlight decode hot path.

This module only makes inputs.  It holds none of the method's arithmetic (no
hashing MLP, no Hamming distance, no top-k, no attention) and is the one module
that both the CPU oracle's tests and the HIP path's tests / bench may import.

Every value is a pure function of (seed, tensor tag, element position):

  * a 32-bit integer mixer turns (seed, tag, 64-bit element counter) into 32
    pseudo-random bits using integer multiply / xor / shift only;
  * the top 16 bits index a 65536-entry table of standard-normal quantiles
    (mid-point rule), so a "normal" draw is an integer hash plus one gather.

Integer ops and gathers give bit-identical results in torch on the CPU and on
the GPU, so a tensor can be produced on the device at full size while the CPU
side regenerates just the rows it needs (row-addressable).  The table itself is
computed once per process on the CPU (fp64 -> fp32) and copied to the device.

The workload follows the paper's remark (Sec. 3.2, MLP hashing paragraph, and
the introduction) that queries and keys sit in two narrow, nearly orthogonal
cones: key = 0.8*mu_k + eps, query = 0.8*mu_q + eps with mu_k, mu_q orthogonal
unit vectors per head and eps ~ N(0, I).  "Needle" keys are exact copies of the
head's query vector at seeded distinct positions.  Hash weights are N(0, 0.05).
These tensors stand in for LLaMA-2-7B / LLaMA-3-8B shaped attention layers run
on long documents, which are not available here.
"""
from __future__ import annotations

import dataclasses
from typing import Dict, List, Optional

import numpy as np
import torch

_M32 = 0xFFFFFFFF
_TABLE_BITS = 16

# tensor tags (any distinct small integers)
TAG_K, TAG_V, TAG_Q, TAG_W1, TAG_B1, TAG_W2 = 1, 2, 3, 4, 5, 6
TAG_MU, TAG_NEEDLE, TAG_CODES, TAG_IDX = 7, 8, 9, 10

_table_cache: Dict[str, torch.Tensor] = {}


def _quantile_table(device: torch.device) -> torch.Tensor:
    """65536 standard-normal quantiles at the bin mid-points, as fp32."""
    key = str(device)
    if key not in _table_cache:
        if "cpu" not in _table_cache:
            from scipy.special import ndtri

            n = 1 << _TABLE_BITS
            p = (np.arange(n, dtype=np.float64) + 0.5) / n
            _table_cache["cpu"] = torch.from_numpy(ndtri(p).astype(np.float32))
        _table_cache[key] = _table_cache["cpu"].to(device)
    return _table_cache[key]


def _mix32(x: torch.Tensor) -> torch.Tensor:
    """A 32-bit avalanche mixer on int64 tensors holding values in [0, 2^32)."""
    x = x ^ (x >> 16)
    x = (x * 0x7FEB352D) & _M32
    x = x ^ (x >> 15)
    x = (x * 0x846CA68B) & _M32
    x = x ^ (x >> 16)
    return x


def random_bits32(seed: int, tag: int, start: int, count: int,
                  device="cpu") -> torch.Tensor:
    """32 pseudo-random bits for element counters start .. start+count-1 (int64 in [0,2^32))."""
    device = torch.device(device)
    e = torch.arange(start, start + count, dtype=torch.int64, device=device)
    lo = e & _M32
    hi = (e >> 32) & _M32
    key = ((seed & _M32) * 0x9E3779B1 + (tag & _M32) * 0x85EBCA77 + 0x165667B1) & _M32
    x = _mix32(lo ^ key)
    x = _mix32((x + hi * 0xC2B2AE3D + ((key * 0x27D4EB2F) & _M32)) & _M32)
    return x


def normal(seed: int, tag: int, start: int, count: int, device="cpu") -> torch.Tensor:
    """count standard-normal fp32 draws for element counters start .. start+count-1."""
    bits = random_bits32(seed, tag, start, count, device)
    return _quantile_table(torch.device(device))[bits >> (32 - _TABLE_BITS)]


def uniform_int(seed: int, tag: int, start: int, count: int, modulus: int,
                device="cpu") -> torch.Tensor:
    return random_bits32(seed, tag, start, count, device) % modulus


def rotation_matrix(seed: int, tag: int, start: int, d: int) -> torch.Tensor:
    """A d x d rotation (orthogonal, determinant +1) as the paper's appendix on LSH weight
    initialisation builds it: QR decomposition of a matrix of independent N(0,1) entries (here by
    modified Gram-Schmidt in float64 on the host, so that the result does not depend on a linear
    algebra library), the first column negated if the determinant is negative.  float32, rows are
    the hyperplane normals."""
    a = normal(seed, tag, start, d * d).double().view(d, d)
    q = torch.zeros(d, d, dtype=torch.float64)
    for j in range(d):
        v = a[:, j].clone()
        for _ in range(2):                       # second pass: re-orthogonalisation
            v = v - q[:, :j] @ (q[:, :j].T @ v)
        q[:, j] = v / v.norm()
    if torch.linalg.det(q) < 0:
        q[:, 0] = -q[:, 0]
    return q.float()


_TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16}


@dataclasses.dataclass(frozen=True)
class Config:
    """One decode-step workload (shapes follow LLaMA-style attention layers)."""
    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    n_tokens: int
    code_bits: int
    hidden: int
    topk: int
    kv_dtype: str            # "f32" | "bf16"
    weight_dtype: str        # "f32" | "bf16"
    needles: int             # per query head
    seed: int
    head_dim: int = 128
    extra_tokens: int = 0    # room for appended keys (cache growth)
    lsh_init: str = "gaussian"   # linear hash (hidden == 0) only: "gaussian" | "rotation"

    @property
    def max_tokens(self) -> int:
        return self.n_tokens + self.extra_tokens

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def words(self) -> int:
        return self.code_bits // 32

    def scaled(self, **kw) -> "Config":
        return dataclasses.replace(self, **kw)


def _cfg(i, **kw) -> Config:
    return Config(seed=0x5107 + i, **kw)


# The five workloads the build is measured on.  k is 2 % of the context rounded
# up for C2/C3, 1 % for C5, and fixed at 128 / 2048 for C1 / C4.
CONFIGS: Dict[str, Config] = {
    "C1": _cfg(1, name="C1", batch=1, n_q_heads=1, n_kv_heads=1, n_tokens=4096,
               code_bits=128, hidden=256, topk=128, kv_dtype="f32", weight_dtype="f32", needles=8),
    "C2": _cfg(2, name="C2", batch=1, n_q_heads=32, n_kv_heads=32, n_tokens=32768,
               code_bits=128, hidden=256, topk=656, kv_dtype="bf16", weight_dtype="bf16", needles=16),
    "C3": _cfg(3, name="C3", batch=1, n_q_heads=32, n_kv_heads=32, n_tokens=524288,
               code_bits=128, hidden=256, topk=10486, kv_dtype="bf16", weight_dtype="bf16", needles=64),
    "C4": _cfg(4, name="C4", batch=16, n_q_heads=32, n_kv_heads=8, n_tokens=131072,
               code_bits=256, hidden=512, topk=2048, kv_dtype="bf16", weight_dtype="bf16", needles=4),
    "C5-512": _cfg(5, name="C5-512", batch=4, n_q_heads=32, n_kv_heads=32, n_tokens=1048576,
                   code_bits=512, hidden=1024, topk=10486, kv_dtype="bf16", weight_dtype="bf16",
                   needles=8, extra_tokens=64),
    "C5-128": _cfg(5, name="C5-128", batch=4, n_q_heads=32, n_kv_heads=32, n_tokens=1048576,
                   code_bits=128, hidden=256, topk=10486, kv_dtype="bf16", weight_dtype="bf16",
                   needles=8, extra_tokens=64),
    # Not one of the five: the attention layout of Qwen2.5-7B (28 query heads on 4 key-value heads,
    # groups of seven), the model of the paper's efficiency experiments, at its 128K context.
    "Q7-128K": _cfg(7, name="Q7-128K", batch=1, n_q_heads=28, n_kv_heads=4, n_tokens=131072,
                    code_bits=128, hidden=256, topk=2622, kv_dtype="bf16", weight_dtype="bf16", needles=4),
}


class Workload:
    """Row-addressable tensors of one Config.  Small tensors are built eagerly on the CPU."""

    def __init__(self, cfg: Config):
        assert cfg.n_q_heads % cfg.n_kv_heads == 0
        self.cfg = cfg
        c = cfg
        d = c.head_dim
        self.kv_t = _TORCH_DTYPE[c.kv_dtype]
        self.w_t = _TORCH_DTYPE[c.weight_dtype]
        # cone axes: mu_k per (b, kv head); mu_q per (b, q head), orthogonal to its kv head's mu_k
        g = normal(c.seed, TAG_MU, 0, c.batch * (c.n_kv_heads + c.n_q_heads) * d).double()
        g = g.view(c.batch, c.n_kv_heads + c.n_q_heads, d)
        mu_k = g[:, :c.n_kv_heads]
        mu_k = mu_k / mu_k.norm(dim=-1, keepdim=True)
        mu_q = g[:, c.n_kv_heads:]
        mk = mu_k.repeat_interleave(c.group, dim=1)
        mu_q = mu_q - (mu_q * mk).sum(-1, keepdim=True) * mk
        mu_q = mu_q / mu_q.norm(dim=-1, keepdim=True)
        self.center_k = (0.8 * mu_k).float().contiguous()      # [B, Hkv, d]
        self.center_q = (0.8 * mu_q).float().contiguous()      # [B, Hq, d]
        eps = normal(c.seed, TAG_Q, 0, c.batch * c.n_q_heads * d).view(c.batch, c.n_q_heads, d)
        self.q = (self.center_q + eps).to(self.kv_t).contiguous()  # [B, Hq, d]
        # needle positions: [B, Hq, needles], distinct within each (b, kv head)
        self.needle_pos = self._needle_positions()

    # ---------------------------------------------------------------- weights
    def hash_weights(self, device="cpu"):
        """W1 [Hkv, h, d], b1 [Hkv, h], W2 [Hkv, L, h]; with hidden == 0, W1 is R [Hkv, L, d]."""
        c = self.cfg
        d, h, L = c.head_dim, c.hidden, c.code_bits
        if h == 0 and c.lsh_init == "rotation":
            # Angular LSH initialised with rotation matrices (appendix "LSH Weight Initialization"):
            # a code longer than d bits takes L / d independent rotations side by side.
            assert L % d == 0, "rotation init needs code_bits to be a multiple of head_dim"
            blocks = [rotation_matrix(c.seed, TAG_W1, (hk * (L // d) + j) * d * d, d)
                      for hk in range(c.n_kv_heads) for j in range(L // d)]
            w1 = torch.stack(blocks).view(c.n_kv_heads, L, d)
            return (w1.to(self.w_t).contiguous().to(device), None, None)
        if h == 0:
            w1 = 0.05 * normal(c.seed, TAG_W1, 0, c.n_kv_heads * L * d, device)
            return (w1.view(c.n_kv_heads, L, d).to(self.w_t).contiguous(), None, None)
        w1 = 0.05 * normal(c.seed, TAG_W1, 0, c.n_kv_heads * h * d, device)
        b1 = 0.05 * normal(c.seed, TAG_B1, 0, c.n_kv_heads * h, device)
        w2 = 0.05 * normal(c.seed, TAG_W2, 0, c.n_kv_heads * L * h, device)
        return (w1.view(c.n_kv_heads, h, d).to(self.w_t).contiguous(),
                b1.view(c.n_kv_heads, h).to(self.w_t).contiguous(),
                w2.view(c.n_kv_heads, L, h).to(self.w_t).contiguous())

    # ---------------------------------------------------------------- needles
    def _needle_positions(self) -> torch.Tensor:
        c = self.cfg
        out = torch.zeros(c.batch, c.n_q_heads, max(c.needles, 1), dtype=torch.int64)
        if c.needles == 0:
            return out[:, :, :0]
        per_kv = c.needles * c.group
        assert per_kv <= c.n_tokens
        for b in range(c.batch):
            for hk in range(c.n_kv_heads):
                stream = (b * c.n_kv_heads + hk) * (1 << 20)
                seen: List[int] = []
                off = 0
                while len(seen) < per_kv:
                    cand = uniform_int(c.seed, TAG_NEEDLE, stream + off, 4 * per_kv, c.n_tokens).tolist()
                    off += 4 * per_kv
                    for p in cand:
                        if p not in seen:
                            seen.append(p)
                            if len(seen) == per_kv:
                                break
                for j in range(c.group):
                    out[b, hk * c.group + j] = torch.tensor(seen[j * c.needles:(j + 1) * c.needles])
        return out

    # ---------------------------------------------------------------- K / V rows
    def kv_rows(self, which: str, b: int, hk: int, t0: int, n: int, device="cpu") -> torch.Tensor:
        """Rows [t0, t0+n) of K or V for (b, kv head): [n, d] in kv dtype.  Row t of the
        virtual [B, Hkv, max_tokens, d] tensor uses element counters ((b*Hkv+hk)*max_tokens+t)*d+c."""
        c = self.cfg
        d = c.head_dim
        base = ((b * c.n_kv_heads + hk) * c.max_tokens + t0) * d
        if which == "V":
            return normal(c.seed, TAG_V, base, n * d, device).view(n, d).to(self.kv_t)
        assert which == "K"
        rows = normal(c.seed, TAG_K, base, n * d, device).view(n, d)
        rows = (rows + self.center_k[b, hk].to(device)).to(self.kv_t)
        for j in range(c.group):
            hq = hk * c.group + j
            pos = self.needle_pos[b, hq]
            sel = pos[(pos >= t0) & (pos < t0 + n)]
            if sel.numel():
                rows[(sel - t0).to(device)] = self.q[b, hq].to(device)
        return rows

    def materialize(self, which: str, device, chunk_rows: int = 1 << 20) -> torch.Tensor:
        """The whole [B, Hkv, max_tokens, d] tensor on `device`, generated chunk by chunk."""
        c = self.cfg
        out = torch.empty(c.batch, c.n_kv_heads, c.max_tokens, c.head_dim, dtype=self.kv_t, device=device)
        for b in range(c.batch):
            for hk in range(c.n_kv_heads):
                for t0 in range(0, c.max_tokens, chunk_rows):
                    n = min(chunk_rows, c.max_tokens - t0)
                    out[b, hk, t0:t0 + n] = self.kv_rows(which, b, hk, t0, n, device)
        return out

    # ---------------------------------------------------------------- synthetic codes
    def synthetic_codes(self, b: int, hk: int, t0: int, n: int, device="cpu") -> torch.Tensor:
        """Packed codes drawn directly (not through the hash MLP), [n, W] int32 bit patterns.
        Each bit is 1 with a per-(head, bit) probability in {1/8 .. 7/8}, which concentrates the
        Hamming distances in a narrow band the way codes of a cone of keys do.  Used where a
        full-size select has to be checked without hashing every key on the CPU."""
        c = self.cfg
        W = c.words
        base = ((b * c.n_kv_heads + hk) * c.max_tokens + t0) * c.code_bits
        r = random_bits32(c.seed, TAG_CODES, base, n * c.code_bits, device) >> 29       # 0..7
        bias = uniform_int(c.seed, TAG_CODES + 100, (b * c.n_kv_heads + hk) * c.code_bits,
                           c.code_bits, 7, device) + 1                                    # 1..7
        bits = (r.view(n, c.code_bits) < bias).to(torch.int64)                             # [n, L]
        sh = torch.arange(32, dtype=torch.int64, device=device)
        words = (bits.view(n, W, 32) << sh).sum(-1)                                        # [n, W]
        words = torch.where(words >= (1 << 31), words - (1 << 32), words)
        return words.to(torch.int32)
