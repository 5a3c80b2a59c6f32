"""Thin ctypes binding of libspotlight.so (include/spotlight.h).  Argument marshalling only:
every step of the path runs in the HIP kernels.  torch supplies device memory and the stream.

There is no fallback: if the library has not been built, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import math
import os
from typing import Optional, Tuple

import torch

from . import build as _build

F32, BF16 = 0, 1
OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_HIP, ERR_TOO_LARGE = 0, -1, -2, -3, -4, -5
NOALLOC_SCRATCH_BYTES = 32 << 20
STAGES = ("hash_keys", "hash_query", "score", "select", "attend", "merge", "step_small")

# every symbol include/spotlight.h declares
SYMBOLS = (
    "spotlight_validate_config", "spotlight_workspace_bytes", "spotlight_create", "spotlight_destroy",
    "spotlight_set_stream", "spotlight_strerror", "spotlight_hash_keys", "spotlight_retrieve_topk",
    "spotlight_sparse_decode", "spotlight_decode_step", "spotlight_prepack_weights", "spotlight_profile_enable",
    "spotlight_profile_read", "spotlight_build_id", "spotlight_set_option", "spotlight_bulk_hash_audit_read",
    "spotlight_decode_step_noalloc",
)
OPT_BULK_HASH_MATRIX_CORES, OPT_BULK_HASH_AUDIT, OPT_STEP_SINGLE_LAUNCH = 0, 1, 2


class Config(C.Structure):
    _fields_ = [
        ("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
        ("code_bits", C.c_int32), ("hidden", C.c_int32), ("max_tokens", C.c_int64), ("max_topk", C.c_int32),
        ("kv_dtype", C.c_int32), ("weight_dtype", C.c_int32), ("stream", C.c_void_p),
    ]


class HashWeights(C.Structure):
    _fields_ = [("w1", C.c_void_p), ("b1", C.c_void_p), ("w2", C.c_void_p)]


def _load() -> C.CDLL:
    path = _build.LIB
    if not os.path.exists(path):
        raise ImportError(
            f"{path} is missing: build the HIP library first "
            "(python -c 'import __graft_entry__ as g; g.build()' or python paper_2508_19740_amd/build.py)")
    lib = C.CDLL(path)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    lib.spotlight_validate_config.argtypes = [C.POINTER(Config)]
    lib.spotlight_workspace_bytes.argtypes = [C.POINTER(Config)]
    lib.spotlight_workspace_bytes.restype = C.c_size_t
    lib.spotlight_create.argtypes = [C.POINTER(vp), C.POINTER(Config)]
    lib.spotlight_destroy.argtypes = [vp]
    lib.spotlight_set_stream.argtypes = [vp, vp]
    lib.spotlight_strerror.argtypes = [C.c_int]
    lib.spotlight_strerror.restype = C.c_char_p
    lib.spotlight_hash_keys.argtypes = [vp, vp, C.POINTER(HashWeights), i64, i64, vp]
    lib.spotlight_retrieve_topk.argtypes = [vp, vp, C.POINTER(HashWeights), vp, i64, i32, vp, vp, vp]
    lib.spotlight_sparse_decode.argtypes = [vp, vp, vp, vp, vp, i32, C.c_float, vp]
    lib.spotlight_decode_step.argtypes = [vp, vp, vp, vp, C.POINTER(HashWeights), vp, i64, i32, i32, i32,
                                          C.c_float, vp, vp]
    lib.spotlight_decode_step_noalloc.argtypes = [C.POINTER(Config), vp, vp, vp, C.POINTER(HashWeights), vp, i64, i32,
                                                  i32, i32, C.c_float, vp, vp]
    lib.spotlight_prepack_weights.argtypes = [vp, C.POINTER(HashWeights)]
    lib.spotlight_profile_enable.argtypes = [vp, C.c_int]
    lib.spotlight_profile_read.argtypes = [vp, C.c_int, C.POINTER(C.c_double), C.POINTER(i64)]
    lib.spotlight_build_id.argtypes = []
    lib.spotlight_build_id.restype = C.c_char_p
    lib.spotlight_set_option.argtypes = [vp, C.c_int, C.c_int]
    lib.spotlight_bulk_hash_audit_read.argtypes = [vp, C.POINTER(i64), C.POINTER(i64), C.POINTER(i64),
                                                   C.POINTER(C.c_double), C.POINTER(C.c_double)]
    return lib


lib = _load()


class SpotlightError(RuntimeError):
    def __init__(self, rc: int, what: str):
        super().__init__(f"{what}: {lib.spotlight_strerror(rc).decode()} ({rc})")
        self.rc = rc


def _dtype_code(t: torch.dtype) -> int:
    if t == torch.float32:
        return F32
    if t == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t}")


def make_config(batch, n_q_heads, n_kv_heads, code_bits, hidden, max_tokens, max_topk,
                kv_dtype=torch.bfloat16, weight_dtype=torch.bfloat16, head_dim=128, stream=None) -> Config:
    return Config(batch, n_q_heads, n_kv_heads, head_dim, code_bits, hidden, max_tokens, max_topk,
                  _dtype_code(kv_dtype), _dtype_code(weight_dtype), stream)


def validate_config(cfg: Config) -> int:
    return lib.spotlight_validate_config(C.byref(cfg))


def workspace_bytes(cfg: Config) -> int:
    return lib.spotlight_workspace_bytes(C.byref(cfg))


def build_id() -> str:
    """Hash of the sources the loaded library was compiled from."""
    return lib.spotlight_build_id().decode().split("=", 1)[1]


class Spotlight:
    """One context = one layer shape.  Methods mirror the C entry points; tensors are checked for
    device, dtype, contiguity and shape on the host before the call."""

    def __init__(self, batch, n_q_heads, n_kv_heads, code_bits, hidden, max_tokens, max_topk,
                 kv_dtype=torch.bfloat16, weight_dtype=torch.bfloat16, head_dim=128, device="cuda:0"):
        self.device = torch.device(device)
        if self.device.type != "cuda":
            raise ValueError("Spotlight needs a GPU device")
        self.kv_dtype, self.weight_dtype = kv_dtype, weight_dtype
        self.B, self.Hq, self.Hkv, self.d = batch, n_q_heads, n_kv_heads, head_dim
        self.L, self.W, self.h = code_bits, code_bits // 32, hidden
        self.Nmax, self.max_topk = max_tokens, max_topk
        with torch.cuda.device(self.device):
            stream = torch.cuda.current_stream(self.device).cuda_stream
            self.cfg = make_config(batch, n_q_heads, n_kv_heads, code_bits, hidden, max_tokens, max_topk,
                                   kv_dtype, weight_dtype, head_dim, stream)
            h = C.c_void_p()
            rc = lib.spotlight_create(C.byref(h), C.byref(self.cfg))
        if rc != OK:
            raise SpotlightError(rc, "spotlight_create")
        self._h = h

    def close(self):
        if getattr(self, "_h", None):
            lib.spotlight_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ------------------------------------------------------------------ helpers
    def _chk(self, t: torch.Tensor, shape, dtype, name):
        if t.device != self.device or not t.is_contiguous() or t.dtype != dtype or tuple(t.shape) != tuple(shape):
            raise ValueError(f"{name}: want contiguous {dtype} {tuple(shape)} on {self.device}, "
                             f"got {t.dtype} {tuple(t.shape)} on {t.device}")
        return t.data_ptr()

    def _weights(self, w1, b1, w2) -> HashWeights:
        if self.h > 0:
            return HashWeights(self._chk(w1, (self.Hkv, self.h, self.d), self.weight_dtype, "w1"),
                               self._chk(b1, (self.Hkv, self.h), self.weight_dtype, "b1"),
                               self._chk(w2, (self.Hkv, self.L, self.h), self.weight_dtype, "w2"))
        return HashWeights(self._chk(w1, (self.Hkv, self.L, self.d), self.weight_dtype, "w1"), None, None)

    def _sync_stream(self):
        s = torch.cuda.current_stream(self.device).cuda_stream
        if s != self.cfg.stream:
            self.cfg.stream = s
            lib.spotlight_set_stream(self._h, s)

    def set_option(self, option: int, value: int):
        rc = lib.spotlight_set_option(self._h, option, value)
        if rc != OK:
            raise SpotlightError(rc, "spotlight_set_option")

    def bulk_hash_audit_read(self) -> dict:
        """Totals of the audited matrix-core bulk hash since the last read (and clears them)."""
        n, li, wr = C.c_int64(), C.c_int64(), C.c_int64()
        ratio, eps = C.c_double(), C.c_double()
        rc = lib.spotlight_bulk_hash_audit_read(self._h, C.byref(n), C.byref(li), C.byref(wr), C.byref(ratio), C.byref(eps))
        if rc != OK:
            raise SpotlightError(rc, "spotlight_bulk_hash_audit_read")
        return {"outputs": n.value, "listed": li.value, "wrong": wr.value, "max_ratio": ratio.value, "eps": eps.value}

    # ------------------------------------------------------------------ entry points
    def prepack_weights(self, w1=None, b1=None, w2=None):
        """Copy the hash weights into the kernel's read order (all None: drop the copy)."""
        self._sync_stream()
        if w1 is None:
            rc = lib.spotlight_prepack_weights(self._h, None)
        else:
            w = self._weights(w1, b1, w2)
            rc = lib.spotlight_prepack_weights(self._h, C.byref(w))
        if rc != OK:
            raise SpotlightError(rc, "spotlight_prepack_weights")
        # The library recognises the arrays its copy was made from by their addresses.  Holding the
        # tensors here keeps those addresses from being freed and handed to other weights while the
        # copy is in use.  (An update of the arrays IN PLACE still needs a new prepack_weights call.)
        self._packed_from = None if w1 is None else (w1, b1, w2)

    def hash_keys(self, K, w1, b1, w2, t0: int, n_new: int, codes):
        self._sync_stream()
        kp = self._chk(K, (self.B, self.Hkv, self.Nmax, self.d), self.kv_dtype, "K")
        cp = self._chk(codes, (self.B, self.Hkv, self.Nmax, self.W), torch.int32, "codes")
        w = self._weights(w1, b1, w2)
        rc = lib.spotlight_hash_keys(self._h, kp, C.byref(w), t0, n_new, cp)
        if rc != OK:
            raise SpotlightError(rc, "spotlight_hash_keys")
        return codes

    def retrieve_topk(self, q, w1, b1, w2, codes, n_tokens: int, k: int, out_idx=None,
                      out_qcode=None, out_dist=None):
        self._sync_stream()
        qp = self._chk(q, (self.B, self.Hq, self.d), self.kv_dtype, "q")
        cp = self._chk(codes, (self.B, self.Hkv, self.Nmax, self.W), torch.int32, "codes")
        w = self._weights(w1, b1, w2)
        if not (isinstance(k, int) and isinstance(n_tokens, int)):
            raise TypeError("k and n_tokens are ints")
        if out_idx is None:
            out_idx = torch.empty(self.B, self.Hq, max(k, 0), dtype=torch.int32, device=self.device)
        ip = self._chk(out_idx, (self.B, self.Hq, k), torch.int32, "out_idx")
        qcp = None if out_qcode is None else self._chk(out_qcode, (self.B, self.Hq, self.W), torch.int32, "out_qcode")
        dp = None if out_dist is None else self._chk(out_dist, (self.B, self.Hq, n_tokens), torch.int16, "out_dist")
        rc = lib.spotlight_retrieve_topk(self._h, qp, C.byref(w), cp, n_tokens, k, ip, qcp, dp)
        if rc != OK:
            raise SpotlightError(rc, "spotlight_retrieve_topk")
        return out_idx

    def sparse_decode(self, q, K, V, idx, scale: Optional[float] = None, out=None):
        self._sync_stream()
        qp = self._chk(q, (self.B, self.Hq, self.d), self.kv_dtype, "q")
        kp = self._chk(K, (self.B, self.Hkv, self.Nmax, self.d), self.kv_dtype, "K")
        vp = self._chk(V, (self.B, self.Hkv, self.Nmax, self.d), self.kv_dtype, "V")
        if idx.dim() != 3:
            raise ValueError("idx: want [B, Hq, k]")
        k = idx.shape[-1]
        ip = self._chk(idx, (self.B, self.Hq, k), torch.int32, "idx")
        if out is None:
            out = torch.empty(self.B, self.Hq, self.d, dtype=torch.float32, device=self.device)
        op = self._chk(out, (self.B, self.Hq, self.d), torch.float32, "out")
        if scale is None:
            scale = 1.0 / math.sqrt(self.d)
        rc = lib.spotlight_sparse_decode(self._h, qp, kp, vp, ip, k, float(scale), op)
        if rc != OK:
            raise SpotlightError(rc, "spotlight_sparse_decode")
        return out

    def decode_step(self, q, K, V, w1, b1, w2, codes, n_tokens: int, k: int, n_sink: int = 0, n_local: int = 0,
                    scale: Optional[float] = None, out_idx=None, out=None):
        """Hash the key at row n_tokens-1 into codes, retrieve (first n_sink / last n_local tokens
        forced), attend: one C call, five kernel launches.  Returns (idx, out)."""
        self._sync_stream()
        qp = self._chk(q, (self.B, self.Hq, self.d), self.kv_dtype, "q")
        kp = self._chk(K, (self.B, self.Hkv, self.Nmax, self.d), self.kv_dtype, "K")
        vp = self._chk(V, (self.B, self.Hkv, self.Nmax, self.d), self.kv_dtype, "V")
        cp = self._chk(codes, (self.B, self.Hkv, self.Nmax, self.W), torch.int32, "codes")
        w = self._weights(w1, b1, w2)
        if not all(isinstance(v, int) for v in (k, n_tokens, n_sink, n_local)):
            raise TypeError("k, n_tokens, n_sink and n_local are ints")
        if out_idx is None:
            out_idx = torch.empty(self.B, self.Hq, max(k, 0), dtype=torch.int32, device=self.device)
        ip = self._chk(out_idx, (self.B, self.Hq, k), torch.int32, "out_idx")
        if out is None:
            out = torch.empty(self.B, self.Hq, self.d, dtype=torch.float32, device=self.device)
        op = self._chk(out, (self.B, self.Hq, self.d), torch.float32, "out")
        if scale is None:
            scale = 1.0 / math.sqrt(self.d)
        rc = lib.spotlight_decode_step(self._h, qp, kp, vp, C.byref(w), cp, n_tokens, k, n_sink, n_local,
                                       float(scale), ip, op)
        if rc != OK:
            raise SpotlightError(rc, "spotlight_decode_step")
        return out_idx, out

    # ------------------------------------------------------------------ stage timing
    def profile_enable(self, on: bool = True):
        rc = lib.spotlight_profile_enable(self._h, 1 if on else 0)
        if rc != OK:
            raise SpotlightError(rc, "spotlight_profile_enable")

    def profile_read(self) -> dict:
        """{stage name: (total milliseconds, launches)} since profiling was enabled."""
        out = {}
        for i, name in enumerate(STAGES):
            ms, n = C.c_double(), C.c_int64()
            rc = lib.spotlight_profile_read(self._h, i, C.byref(ms), C.byref(n))
            if rc != OK:
                raise SpotlightError(rc, "spotlight_profile_read")
            out[name] = (ms.value, n.value)
        return out


def spotlight_decode_step_noalloc(cfg: Config, q, K, V, w1, b1, w2, codes, n_tokens: int, k: int, n_sink: int,
                                  n_local: int, scale: float, out_idx, out) -> int:
    """The decode step without a context: the library's fixed scratch buffer is the workspace and
    nothing is allocated, here or in the library, so the caller brings out_idx and out.  Pointers
    only: the tensors must be contiguous device tensors of the shapes spotlight_decode_step takes.
    Returns the C return code."""
    w = HashWeights(w1.data_ptr(), None if b1 is None else b1.data_ptr(), None if w2 is None else w2.data_ptr())
    return lib.spotlight_decode_step_noalloc(C.byref(cfg), q.data_ptr(), K.data_ptr(), V.data_ptr(), C.byref(w),
                                             codes.data_ptr(), n_tokens, k, n_sink, n_local, float(scale),
                                             out_idx.data_ptr(), out.data_ptr())


# flat functions named like the C entry points
def spotlight_hash_keys(ctx: Spotlight, K, w1, b1, w2, t0, n_new, codes):
    return ctx.hash_keys(K, w1, b1, w2, t0, n_new, codes)


def spotlight_retrieve_topk(ctx: Spotlight, q, w1, b1, w2, codes, n_tokens, k, **kw):
    return ctx.retrieve_topk(q, w1, b1, w2, codes, n_tokens, k, **kw)


def spotlight_sparse_decode(ctx: Spotlight, q, K, V, idx, scale=None, out=None):
    return ctx.sparse_decode(q, K, V, idx, scale, out)


def spotlight_prepack_weights(ctx: Spotlight, w1=None, b1=None, w2=None):
    return ctx.prepack_weights(w1, b1, w2)


def spotlight_decode_step(ctx: Spotlight, q, K, V, w1, b1, w2, codes, n_tokens, k, n_sink=0, n_local=0, **kw):
    return ctx.decode_step(q, K, V, w1, b1, w2, codes, n_tokens, k, n_sink, n_local, **kw)
