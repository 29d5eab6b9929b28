"""MI355X-native QuIVer query hot path: Sign-Magnitude encode, code-space beam search, float32 rerank.

The work is done by ``libquiver_hip.so`` (HIP, gfx950; C ABI in ``include/quiver.h``); this package
is its thin binding.
"""
from .binding import (EMPTY, MAX_EF, STATUS_BAD_EDGE, STATUS_NONFINITE, STATUS_VISITED_FULL, Index, QuiverError,
                      SearchOutput, Timer, bq_distance, bq_scan, build_graph, topk_overlap, code_words, encode, gather_probe, from_numpy_u32, from_numpy_u64, search,
                      search_workspace_bytes, to_numpy_u32, to_numpy_u64)

__all__ = ["EMPTY", "MAX_EF", "STATUS_BAD_EDGE", "STATUS_NONFINITE", "STATUS_VISITED_FULL", "Index", "QuiverError",
           "SearchOutput", "Timer", "bq_distance", "bq_scan", "build_graph", "topk_overlap", "code_words", "encode", "gather_probe", "from_numpy_u32", "from_numpy_u64",
           "search", "search_workspace_bytes", "to_numpy_u32", "to_numpy_u64"]
