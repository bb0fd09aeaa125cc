"""MI355X-native relay-boundary KV compression (headwise eviction + Orthogonal BackFill).

Thin Python binding over libobf_relay.so (HIP kernels behind a C ABI).  Every step of the
path runs in the library's kernels; this package only marshals arguments.  There is no CPU
fallback: without the built library the calls raise.
"""
from .binding import (  # noqa: F401
    DIAG_DTYPE,
    ObfError,
    backfill,
    compress_relay,
    gather,
    lib_path,
    load_library,
    refine_boundary,
    score,
    select_topk,
    shape_of,
    workspace_bytes,
)
