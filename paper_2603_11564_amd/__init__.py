"""DapQ eviction scoring for MI355X: a thin ctypes binding over libdapq.so (hand-written HIP, gfx950).

Only argument marshalling happens here; every step of the path runs in the library's kernels.
There is no fallback: if libdapq.so is missing, importing `paper_2603_11564_amd.binding` raises.
"""
from .binding import (  # noqa: F401
    DapqError, Shape, Qproj, lib_path, load_library, make_shape, workspace_bytes,
    dapq_rope_apply, dapq_score, dapq_score_stats, dapq_score_accumulate, dapq_score_stats_extend, dapq_pool,
    dapq_topk, dapq_pool_topk, dapq_gather, dapq_recall, dapq_decode_attention, dapq_pseudo_tokens, dapq_pseudo_queries, pseudo_queries_workspace_bytes,
    dapq_score_static, score_static_capacity, score_single_launch, topk_workspace_bytes,
)
