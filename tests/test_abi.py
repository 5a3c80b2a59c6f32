"""Host-side checks of the C ABI that need no GPU: the library loads, exports exactly what
include/spotlight.h declares, validates configurations and arguments before any HIP call."""
import ctypes as C
import os
import re
import subprocess

import pytest
import torch

import paper_2508_19740_amd as sp

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "spotlight.h")
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _declared():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(spotlight_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported_and_bound():
    declared = _declared()
    assert declared == sorted(sp.SYMBOLS)
    out = subprocess.run(["nm", "-D", "--defined-only", sp.lib._name], capture_output=True, text=True, check=True).stdout
    exported = set(re.findall(r" T (spotlight_[a-z_]+)", out))
    assert set(declared) <= exported
    for name in declared:
        assert getattr(sp.lib, name) is not None


def test_header_compiles_as_plain_c():
    src = '#include "spotlight.h"\nint main(void){ spotlight_config c; (void)c; return SPOTLIGHT_STAGE_COUNT == 7 ? 0 : 1; }\n'
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-fsyntax-only", "-I", os.path.join(ROOT, "include"),
                    "-x", "c", "-"], input=src, text=True, check=True)


def _cfg(**kw):
    base = dict(batch=1, n_q_heads=32, n_kv_heads=32, code_bits=128, hidden=256, max_tokens=4096, max_topk=128)
    base.update(kw)
    return sp.make_config(**base)


def test_validate_config_accepts_the_five_workloads():
    import workload as wl
    for c in wl.CONFIGS.values():
        cfg = sp.make_config(c.batch, c.n_q_heads, c.n_kv_heads, c.code_bits, c.hidden, c.max_tokens, c.topk)
        assert sp.validate_config(cfg) == sp.OK, c.name
        assert sp.workspace_bytes(cfg) > 0


@pytest.mark.parametrize("kw,rc", [
    (dict(batch=0), sp.ERR_INVALID_ARG),
    (dict(n_q_heads=30, n_kv_heads=8), sp.ERR_INVALID_ARG),      # not a multiple
    (dict(code_bits=100), sp.ERR_INVALID_ARG),
    (dict(code_bits=0), sp.ERR_INVALID_ARG),
    (dict(code_bits=1056), sp.ERR_INVALID_ARG),
    (dict(code_bits=544), sp.ERR_UNSUPPORTED),                   # above 512 only 1024 bits
    (dict(code_bits=1024, n_q_heads=32, n_kv_heads=8), sp.ERR_UNSUPPORTED),   # 1024 bits: at most 2 heads per group
    (dict(hidden=-8), sp.ERR_INVALID_ARG),
    (dict(max_tokens=0), sp.ERR_INVALID_ARG),
    (dict(max_topk=0), sp.ERR_INVALID_ARG),
    (dict(max_topk=5000), sp.ERR_INVALID_ARG),                   # larger than max_tokens
    (dict(head_dim=64), sp.ERR_UNSUPPORTED),
    (dict(n_q_heads=36, n_kv_heads=4), sp.ERR_UNSUPPORTED),      # group of 9
    (dict(hidden=100), sp.ERR_UNSUPPORTED),                      # not a multiple of 8
])
def test_validate_config_rejects(kw, rc):
    cfg = _cfg(**kw)
    assert sp.validate_config(cfg) == rc
    assert sp.workspace_bytes(cfg) == 0
    h = C.c_void_p()
    assert sp.lib.spotlight_create(C.byref(h), C.byref(cfg)) == rc      # rejected before any HIP call
    assert not h.value


def test_workspace_grows_with_the_problem():
    small = sp.workspace_bytes(_cfg(max_tokens=4096))
    big = sp.workspace_bytes(_cfg(max_tokens=1 << 20, max_topk=128))
    assert big > small
    # about one byte per (query head, token) for the candidate lists, plus histograms
    assert big < 32 * (1 << 20) * 2
    # room for one packed copy of the hash weights: about their own size
    wide = sp.workspace_bytes(_cfg(max_tokens=4096, hidden=1024, code_bits=512))
    more_weights = 32 * ((1024 * 128 + 512 * 1024) - (256 * 128 + 128 * 256)) * 2   # bf16, 32 kv heads
    assert more_weights <= wide - small <= more_weights + (1 << 20)


def test_null_arguments_are_rejected_without_a_gpu():
    bad = sp.ERR_INVALID_ARG
    lib = sp.lib
    assert lib.spotlight_create(None, None) == bad
    assert lib.spotlight_validate_config(None) == bad
    assert lib.spotlight_hash_keys(None, None, None, 0, 0, None) == bad
    assert lib.spotlight_retrieve_topk(None, None, None, None, 1, 1, None, None, None) == bad
    assert lib.spotlight_sparse_decode(None, None, None, None, None, 1, 0.1, None) == bad
    assert lib.spotlight_prepack_weights(None, None) == bad
    assert lib.spotlight_profile_enable(None, 1) == bad
    assert lib.spotlight_profile_read(None, 0, None, None) == bad
    assert lib.spotlight_set_stream(None, None) == bad
    assert lib.spotlight_set_option(None, 0, 1) == bad
    assert lib.spotlight_decode_step_noalloc(None, None, None, None, None, None, 1, 1, 0, 0, 0.1, None, None) == bad
    assert lib.spotlight_bulk_hash_audit_read(None, None, None, None, None, None) == bad
    assert lib.spotlight_destroy(None) == sp.OK
    for rc in (0, -1, -2, -3, -4, -5, -99):
        assert lib.spotlight_strerror(rc)


def test_library_records_the_sources_it_was_built_from():
    """The build id inside the library is the hash of the sources in the tree (a stale library is
    rebuilt before the tests start), and the copy read from the file equals the loaded one."""
    from paper_2508_19740_amd import build as hip_build
    assert sp.build_id() == hip_build.source_id() == hip_build.built_id()
    assert not hip_build.stale()


def test_token_budget_matches_the_paper():
    for line in open(os.path.join(GOLDEN, "token_budget.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        n, rate, want = [s.strip() for s in line.split(";")]
        assert sp.token_budget(int(n), float(rate)) == int(want)


def test_binding_needs_a_gpu_device():
    with pytest.raises(ValueError):
        sp.Spotlight(1, 1, 1, 128, 256, 1024, 16, device="cpu")
