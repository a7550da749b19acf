"""MI355X-native TokenSelect hot path: thin Python binding over libtokenselect.so (C ABI, HIP kernels).

Importing this package does not load the library; the first call does, and raises if it is missing.
"""
from .binding import (  # noqa: F401
    TS_BF16, TS_F32, TS_TOPK_FLAT_VOTES, TokenSelectError, Problem, lib_path, load, ts_paged_qk_scores, ts_selcache_check,
    ts_soft_vote, ts_sparse_paged_attn, ts_strerror, ts_topk, ts_version, ts_workspace_bytes,
    ts_workspace_init, ts_debug_set_score_variant, declared_symbols, ts_chunk_row_stats, ts_chunk_soft_vote,
    ts_chunk_mean_query, ts_sum_vote, ts_head_vote, ts_head_vote_scratch_bytes,
    ts_debug_set_topk_path, ts_debug_event_create, ts_debug_event_destroy, ts_debug_event_elapsed_ms,
    ts_debug_set_score_timing_events, ts_paged_qk_codes, ts_soft_vote_bounds, ts_topk_exact, ts_debug_set_codes_path, ts_topk_noalloc,
    ts_paged_qk_scores_checked, ts_paged_qk_codes_checked, ts_soft_vote_ranked, TS_TOPK_VOTE_HIST,
)
