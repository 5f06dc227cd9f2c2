"""MI355X-native verification hot path of SpecExtend (arXiv 2505.20776).

Hybrid Tree Attention + Cross-model Retrieval as hand-written HIP kernels for
gfx950 behind a small C ABI (include/specext.h); this package is the thin
Python binding over it.  PyTorch supplies device memory and streams only.
"""
from .binding import (prefill_attn, attn_materialized, chunk_scores_materialized, materialized_bytes, materialized_ld, accept_greedy, chunk_scores_accepted, commit_tree_kv, SPECEXT_BF16, SPECEXT_F32, SPECEXT_FLAG_PREFIX_ONLY, SPECEXT_FLAG_VALU_PREFIX, SPECEXT_FLAG_FUSED_MERGE, SPECEXT_FLAG_SHORT_WAIT, WORKSPACE_HEADER_BYTES, workspace_init, chunk_scores_select, calib_stream_read, calib_mfma, calib_issue_mix, SPECEXT_MAX_SPLITS, SPECEXT_MAX_TREE, SpecextError,
                      chunk_scores, gather_draft_kv, load_library, make_desc, num_splits, select_chunks,
                      specext_desc, strerror, verify_attn, verify_attn_static, workspace_bytes)

__all__ = ["prefill_attn", "attn_materialized", "chunk_scores_materialized", "materialized_bytes", "materialized_ld", "accept_greedy", "chunk_scores_accepted", "commit_tree_kv", "SPECEXT_BF16", "SPECEXT_F32", "SPECEXT_FLAG_PREFIX_ONLY", "SPECEXT_FLAG_VALU_PREFIX", "SPECEXT_FLAG_FUSED_MERGE", "SPECEXT_FLAG_SHORT_WAIT", "WORKSPACE_HEADER_BYTES", "workspace_init", "chunk_scores_select", "calib_stream_read", "calib_mfma", "calib_issue_mix", "SPECEXT_MAX_SPLITS", "SPECEXT_MAX_TREE", "SpecextError",
           "chunk_scores", "gather_draft_kv", "load_library", "make_desc", "num_splits", "select_chunks",
           "specext_desc", "strerror", "verify_attn", "verify_attn_static", "workspace_bytes"]
