"""MI355X-native QuIVer query hot path: Sign-Magnitude encode, code-space beam search, float32 rerank.

The work is done by ``libquiver_hip.so`` (HIP, gfx950; C ABI in ``include/quiver.h``); this package
is its thin binding.
"""
from .binding import (EMPTY, ENC_SIGN1, ENC_SM, ENC_SQ2, MAX_EF, RERANK_FUSED, RERANK_SEPARATE, RERANK_TAIL, STATUS_BAD_EDGE, STATUS_NONFINITE, STATUS_VISITED_FULL, VISITED_CACHE,
                      VISITED_EXACT, Index, QuiverError, SearchOutput, Timer, bq_distance, bq_scan, build_graph,
                      code_layout, code_words, encode, pad_codes, from_numpy_u32, from_numpy_u64, gather_probe, search,
                      search_static, search_workspace_bytes, split_codes, split_layout, STATIC_SCRATCH_BYTES, to_numpy_u32, to_numpy_u64, topk_overlap)

__all__ = ["EMPTY", "ENC_SIGN1", "ENC_SM", "ENC_SQ2", "MAX_EF", "RERANK_FUSED", "RERANK_SEPARATE", "RERANK_TAIL", "STATUS_BAD_EDGE", "STATUS_NONFINITE", "STATUS_VISITED_FULL", "VISITED_CACHE",
           "VISITED_EXACT", "Index", "QuiverError", "SearchOutput", "Timer", "bq_distance", "bq_scan", "build_graph",
           "code_layout", "code_words", "encode", "pad_codes", "from_numpy_u32", "from_numpy_u64", "gather_probe", "search",
           "search_static", "search_workspace_bytes", "split_codes", "split_layout", "STATIC_SCRATCH_BYTES", "to_numpy_u32", "to_numpy_u64", "topk_overlap"]
