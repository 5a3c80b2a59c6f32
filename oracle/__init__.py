"""ctypes binding of the CPU oracle (oracle/spotlight_oracle.c).

Test infrastructure only: imported by tests/, by __graft_entry__.smoke() and by bench.py's
cpu_baseline leg.  The product package never imports this module.

All tensors are torch CPU tensors (contiguous).  dtype codes: float32 = 0, bfloat16 = 1.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path) or os.path.getmtime(path) < os.path.getmtime(_build.SRC):
            _build.build()
        L = C.CDLL(path)
        L.ref_exp.restype = C.c_float
        L.ref_exp.argtypes = [C.c_float]
        L.ref_silu.restype = C.c_float
        L.ref_silu.argtypes = [C.c_float]
        L.ref_num_threads.restype = C.c_int
        vp, i32, i64, f64 = C.c_void_p, C.c_int, C.c_int64, C.c_double
        L.ref_pack_bits.argtypes = [vp, i64, i32, vp]
        L.ref_hash_rows.argtypes = [vp, i32, i64, i32, vp, vp, vp, i32, i32, i32, vp, vp, vp]
        L.ref_hash_margin_f64.argtypes = [vp, i32, i64, i32, vp, vp, vp, i32, i32, i32, vp, vp]
        L.ref_hamming.argtypes = [vp, vp, i64, i32, vp]
        L.ref_nxor_score.argtypes = [vp, vp, i32]
        L.ref_topk.argtypes = [vp, i64, i32, vp]
        L.ref_sparse_attention.argtypes = [vp, vp, vp, i32, i32, vp, i32, f64, vp]
        L.ref_hash_keys.argtypes = [i32, i32, i32, i32, i32, i64, i32, i32, vp, vp, vp, vp, i64, i64, vp]
        L.ref_retrieve_topk.argtypes = [i32, i32, i32, i32, i32, i32, i64, i32, i32, vp, vp, vp, vp,
                                        vp, i64, i32, vp, vp, vp]
        L.ref_sparse_decode.argtypes = [i32, i32, i32, i32, i64, i32, vp, vp, vp, vp, i32, f64, vp]
        L.ref_topk_forced.argtypes = [vp, i64, i32, i32, i32, vp]
        L.ref_decode_step.argtypes = [i32, i32, i32, i32, i32, i32, i64, i32, i32, vp, vp, vp, vp, vp, vp,
                                      vp, i64, i32, i32, i32, f64, vp, vp]
        _lib = L
    return _lib


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return 0
    if t.dtype == torch.bfloat16:
        return 1
    raise TypeError(f"unsupported dtype {t.dtype}")


def _p(t):
    if t is None:
        return None
    assert t.device.type == "cpu" and t.is_contiguous(), "oracle takes contiguous CPU tensors"
    return t.data_ptr()


def _check(rc: int, what: str):
    if rc != 0:
        raise ValueError(f"oracle {what} failed with code {rc}")


def num_threads() -> int:
    return lib().ref_num_threads()


def exp32(t: float) -> float:
    return lib().ref_exp(t)


def silu32(a: float) -> float:
    return lib().ref_silu(a)


def pack_bits(bits: torch.Tensor) -> torch.Tensor:
    """bits [n, L] uint8 (0/1) -> codes [n, L/32] int32 (uint32 bit patterns)."""
    n, L = bits.shape
    out = torch.empty(n, L // 32, dtype=torch.int32)
    _check(lib().ref_pack_bits(_p(bits), n, L, _p(out)), "pack_bits")
    return out


def hash_rows(x, w1, b1, w2, code_bits: int, want_y: bool = False):
    """x [n, d]; one head's weights w1 [h, d], b1 [h], w2 [L, h] (or w1 = R [L, d], b1 = w2 = None).
    Returns (bits [n, L] uint8, codes [n, L/32] int32[, y [n, L] float32])."""
    n, d = x.shape
    hidden = 0 if w2 is None else w1.shape[0]
    bits = torch.empty(n, code_bits, dtype=torch.uint8)
    codes = torch.empty(n, code_bits // 32, dtype=torch.int32)
    y = torch.empty(n, code_bits, dtype=torch.float32) if want_y else None
    _check(lib().ref_hash_rows(_p(x), _dt(x), n, d, _p(w1), _p(b1), _p(w2), _dt(w1), hidden,
                               code_bits, _p(bits), _p(codes), _p(y)), "hash_rows")
    return (bits, codes, y) if want_y else (bits, codes)


def hash_margin_f64(x, w1, b1, w2, code_bits: int):
    n, d = x.shape
    y = torch.empty(n, code_bits, dtype=torch.float64)
    mag = torch.empty(n, code_bits, dtype=torch.float64)
    _check(lib().ref_hash_margin_f64(_p(x), _dt(x), n, d, _p(w1), _p(b1), _p(w2), _dt(w1),
                                     w1.shape[0], code_bits, _p(y), _p(mag)), "hash_margin_f64")
    return y, mag


def hamming(qcode: torch.Tensor, codes: torch.Tensor) -> torch.Tensor:
    """qcode [W] int32, codes [n, W] int32 -> dist [n] int16 holding 0..L."""
    n, W = codes.shape
    dist = torch.empty(n, dtype=torch.int16)
    _check(lib().ref_hamming(_p(qcode), _p(codes), n, W * 32, _p(dist)), "hamming")
    return dist


def nxor_score(a: torch.Tensor, b: torch.Tensor) -> int:
    return lib().ref_nxor_score(_p(a), _p(b), a.numel() * 32)


def topk(dist: torch.Tensor, k: int) -> torch.Tensor:
    idx = torch.empty(k, dtype=torch.int32)
    _check(lib().ref_topk(_p(dist), dist.numel(), k, _p(idx)), "topk")
    return idx


def topk_forced(dist: torch.Tensor, k: int, n_sink: int, n_local: int) -> torch.Tensor:
    """The first n_sink and last n_local tokens plus the nearest of the others, k in all, ascending."""
    idx = torch.empty(k, dtype=torch.int32)
    _check(lib().ref_topk_forced(_p(dist), dist.numel(), k, n_sink, n_local, _p(idx)), "topk_forced")
    return idx


def sparse_attention(q, K, V, idx, scale: float) -> torch.Tensor:
    """q [d]; K, V [n, d] of one head; idx [k] int32 -> out [d] float32."""
    d = q.numel()
    out = torch.empty(d, dtype=torch.float32)
    _check(lib().ref_sparse_attention(_p(q), _p(K), _p(V), _dt(K), d, _p(idx), idx.numel(),
                                      float(scale), _p(out)), "sparse_attention")
    return out


# ------------------------------------------------------------------ layer-level calls
def hash_keys(K, w1, b1, w2, code_bits: int, t0: int, n_new: int, codes: torch.Tensor):
    """K [B, Hkv, Nmax, d]; codes [B, Hkv, Nmax, W] int32 updated in place for rows [t0, t0+n_new)."""
    B, Hkv, Nmax, d = K.shape
    hidden = 0 if w2 is None else w1.shape[1]
    _check(lib().ref_hash_keys(B, Hkv, d, code_bits, hidden, Nmax, _dt(K), _dt(w1), _p(K), _p(w1),
                               _p(b1), _p(w2), t0, n_new, _p(codes)), "hash_keys")
    return codes


def retrieve_topk(q, w1, b1, w2, codes, n_tokens: int, k: int, want_dist: bool = False):
    """q [B, Hq, d]; codes [B, Hkv, Nmax, W] -> idx [B, Hq, k] int32, qcode [B, Hq, W] int32,
    dist [B, Hq, n_tokens] int16 (or None)."""
    B, Hq, d = q.shape
    _, Hkv, Nmax, W = codes.shape
    hidden = 0 if w2 is None else w1.shape[1]
    idx = torch.empty(B, Hq, k, dtype=torch.int32)
    qcode = torch.empty(B, Hq, W, dtype=torch.int32)
    dist = torch.empty(B, Hq, n_tokens, dtype=torch.int16) if want_dist else None
    _check(lib().ref_retrieve_topk(B, Hq, Hkv, d, W * 32, hidden, Nmax, _dt(q), _dt(w1), _p(q),
                                   _p(w1), _p(b1), _p(w2), _p(codes), n_tokens, k,
                                   _p(idx), _p(qcode), _p(dist)), "retrieve_topk")
    return idx, qcode, dist


def sparse_decode(q, K, V, idx, scale: float) -> torch.Tensor:
    """q [B, Hq, d]; K, V [B, Hkv, Nmax, d]; idx [B, Hq, k] -> out [B, Hq, d] float32."""
    B, Hq, d = q.shape
    _, Hkv, Nmax, _ = K.shape
    k = idx.shape[-1]
    out = torch.empty(B, Hq, d, dtype=torch.float32)
    _check(lib().ref_sparse_decode(B, Hq, Hkv, d, Nmax, _dt(K), _p(q), _p(K), _p(V), _p(idx), k,
                                   float(scale), _p(out)), "sparse_decode")
    return out


def decode_step(q, K, V, w1, b1, w2, codes, n_tokens: int, k: int, n_sink: int, n_local: int, scale: float):
    """One decode step: hash K[:, :, n_tokens-1] into codes (in place), retrieve with forced sink /
    local tokens, attend.  Returns idx [B, Hq, k] int32 and out [B, Hq, d] float32."""
    B, Hq, d = q.shape
    _, Hkv, Nmax, W = codes.shape
    hidden = 0 if w2 is None else w1.shape[1]
    idx = torch.empty(B, Hq, k, dtype=torch.int32)
    out = torch.empty(B, Hq, d, dtype=torch.float32)
    _check(lib().ref_decode_step(B, Hq, Hkv, d, W * 32, hidden, Nmax, _dt(K), _dt(w1), _p(q), _p(K), _p(V),
                                 _p(w1), _p(b1), _p(w2), _p(codes), n_tokens, k, n_sink, n_local,
                                 float(scale), _p(idx), _p(out)), "decode_step")
    return idx, out
