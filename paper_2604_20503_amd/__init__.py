"""MI355X-native verification step of speculative decoding with per-request speculative lengths.

Thin binding over ``libfaser_verify.so`` (hand-written HIP for gfx950).  Every step of the
hot path runs inside the library; this package only marshals arguments.  PyTorch supplies
device memory and streams.  Importing the package does not load the library; the first call
does, and fails loudly if it has not been built (``python paper_2604_20503_amd/build.py``).
"""
from .binding import (  # noqa: F401
    FsrError,
    accept_workspace_bytes,
    attn_path,
    attn_plan,
    attn_workspace_bytes,
    frontier_commit,
    frontier_init,
    frontier_plan,
    hbm_read_probe,
    kv_append,
    kv_append_kv8,
    last_error,
    library_path,
    load_library,
    prune_compact,
    prune_restore,
    prune_scatter,
    spec_accept,
    survivor_compact,
    survivor_mask,
    topk_rank_check,
    verify_attention,
    verify_attention_kv8,
    verify_attention_static,
    version,
)
from .frontier import verify_chunked  # noqa: F401

__all__ = [
    "FsrError", "accept_workspace_bytes", "attn_path", "attn_plan", "attn_workspace_bytes", "frontier_commit", "frontier_init",
    "frontier_plan", "hbm_read_probe", "kv_append", "kv_append_kv8", "last_error", "library_path", "load_library", "prune_compact", "prune_restore", "prune_scatter",
    "spec_accept", "survivor_compact", "survivor_mask", "topk_rank_check", "verify_attention", "verify_attention_kv8", "verify_attention_static", "verify_chunked", "version",
]
