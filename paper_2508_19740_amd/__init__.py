"""Spotlight Attention decode hot path for AMD MI355X (gfx950): hash -> retrieve -> sparse attention.

The work is done by hand-written HIP kernels in libspotlight.so (C ABI: include/spotlight.h);
this package is the thin Python binding over it.  Importing `binding` fails if the library has not
been built; there is no CPU or eager fallback.
"""
from .binding import (  # noqa: F401
    Spotlight, SpotlightError, Config, HashWeights, make_config, validate_config, workspace_bytes,
    spotlight_hash_keys, spotlight_retrieve_topk, spotlight_sparse_decode, spotlight_decode_step,
    spotlight_prepack_weights, lib, SYMBOLS,
    spotlight_decode_step_noalloc, NOALLOC_SCRATCH_BYTES, ERR_TOO_LARGE,
    build_id, OPT_BULK_HASH_MATRIX_CORES, OPT_BULK_HASH_AUDIT, OPT_STEP_SINGLE_LAUNCH,
    STAGES, OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_HIP, F32, BF16,
)
from .policy import token_budget  # noqa: F401,E402
