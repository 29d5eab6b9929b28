"""ctypes front end of the plain CPU oracle (``quiver_oracle.c``).

TEST INFRASTRUCTURE ONLY: the tests, the smoke check and the benchmark's
``cpu_baseline`` leg are the only callers.  Nothing in the product package may
import this module, and this module imports nothing from the product package.

The wrapper does argument marshalling only (numpy arrays in, numpy arrays
out); every step of the method is in the C file, which cites the paper.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "quiver_oracle.c")
_LIB = os.path.join(_HERE, "libquiver_oracle.so")

EMPTY = 0xFFFFFFFF
# encodings: Sign-Magnitude (the method), and the two of the paper's ablation (Sec. 5.5, Table 10)
SM, SIGN1, SQ2 = 0, 1, 2


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP only to spread independent items)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        P = ctypes.c_void_p
        lib.orc_code_words.restype = ctypes.c_int
        lib.orc_code_words.argtypes = [ctypes.c_int]
        lib.orc_encode.restype = ctypes.c_int
        lib.orc_encode.argtypes = [P, ctypes.c_int64, ctypes.c_int, P, ctypes.c_int]
        lib.orc_sm_distance.restype = ctypes.c_uint32
        lib.orc_sm_distance.argtypes = [P, P, ctypes.c_int]
        lib.orc_sm_distance_pairs.restype = ctypes.c_int
        lib.orc_sm_distance_pairs.argtypes = [P, P, P, P, ctypes.c_int64, ctypes.c_int, P]
        lib.orc_rerank.restype = ctypes.c_int
        lib.orc_rerank.argtypes = [P, ctypes.c_int64, ctypes.c_int, P, P, ctypes.c_int, P, ctypes.c_int, P, P, P]
        lib.orc_search.restype = ctypes.c_int
        lib.orc_search.argtypes = [P, ctypes.c_int64, ctypes.c_int64, ctypes.c_int, ctypes.c_int, P, P, P,
                                   ctypes.c_uint32, ctypes.c_int, ctypes.c_int, P, P, P, P, P, P,
                                   ctypes.c_int64, ctypes.c_int]
        lib.orc_bq_scan.restype = ctypes.c_int
        lib.orc_bq_scan.argtypes = [P, ctypes.c_int64, ctypes.c_int, P, ctypes.c_int64, ctypes.c_int, P, P, ctypes.c_int]
        lib.orc_cosine_topk.restype = ctypes.c_int
        lib.orc_cosine_topk.argtypes = [P, ctypes.c_int64, ctypes.c_int, P, ctypes.c_int64, ctypes.c_int, P, ctypes.c_int]
        lib.orc_topk_overlap.restype = ctypes.c_double
        lib.orc_topk_overlap.argtypes = [P, P, ctypes.c_int64, ctypes.c_int]
        lib.orc_build_graph.restype = ctypes.c_int
        lib.orc_build_graph.argtypes = [P, ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_double,
                                        ctypes.c_uint32, ctypes.c_int64, P]
        lib.orc_code_words_enc.restype = ctypes.c_int
        lib.orc_code_words_enc.argtypes = [ctypes.c_int, ctypes.c_int]
        lib.orc_encode_enc.restype = ctypes.c_int
        lib.orc_encode_enc.argtypes = [P, ctypes.c_int64, ctypes.c_int, ctypes.c_int, P, ctypes.c_int]
        lib.orc_distance_enc.restype = ctypes.c_uint32
        lib.orc_distance_enc.argtypes = [P, P, ctypes.c_int, ctypes.c_int]
        lib.orc_distance_pairs_enc.restype = ctypes.c_int
        lib.orc_distance_pairs_enc.argtypes = [P, P, P, P, ctypes.c_int64, ctypes.c_int, ctypes.c_int, P]
        lib.orc_search_enc.restype = ctypes.c_int
        lib.orc_search_enc.argtypes = [ctypes.c_int] + lib.orc_search.argtypes
        lib.orc_bq_scan_enc.restype = ctypes.c_int
        lib.orc_bq_scan_enc.argtypes = [ctypes.c_int] + lib.orc_bq_scan.argtypes
        lib.orc_build_graph_enc.restype = ctypes.c_int
        lib.orc_build_graph_enc.argtypes = [ctypes.c_int] + lib.orc_build_graph.argtypes
        _lib = lib
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


class OracleError(RuntimeError):
    pass


def _check(rc, what):
    if rc != 0:
        raise OracleError(f"{what} failed with code {rc}")


def code_words(d: int, enc: int = SM) -> int:
    return _load().orc_code_words_enc(int(d), int(enc))


def encode(x: np.ndarray, threads: int = 1, enc: int = SM) -> np.ndarray:
    """float32 [n, d] -> uint64 [n, code_words(d, enc)] (SM: sign words, then magnitude words)."""
    x = _c(x, np.float32)
    if x.ndim == 1:
        x = x[None, :]
    n, d = x.shape
    codes = np.zeros((n, code_words(d, enc)), dtype=np.uint64)
    if enc == SM:
        _check(_load().orc_encode(_ptr(x), n, d, _ptr(codes), int(threads)), "orc_encode")
    else:
        _check(_load().orc_encode_enc(_ptr(x), n, d, int(enc), _ptr(codes), int(threads)), "orc_encode_enc")
    return codes


def sm_distance(a: np.ndarray, b: np.ndarray, d: int) -> int:
    a = _c(a, np.uint64)
    b = _c(b, np.uint64)
    assert a.size == code_words(d) and b.size == code_words(d)
    return int(_load().orc_sm_distance(_ptr(a), _ptr(b), int(d)))


def distance(a: np.ndarray, b: np.ndarray, d: int, enc: int) -> int:
    a = _c(a, np.uint64)
    b = _c(b, np.uint64)
    assert a.size == code_words(d, enc) and b.size == code_words(d, enc)
    return int(_load().orc_distance_enc(_ptr(a), _ptr(b), int(d), int(enc)))


def sm_distance_pairs(codes_a, ia, codes_b, ib, d: int, enc: int = SM) -> np.ndarray:
    codes_a = _c(codes_a, np.uint64)
    codes_b = _c(codes_b, np.uint64)
    ia = _c(ia, np.int64)
    ib = _c(ib, np.int64)
    assert ia.shape == ib.shape
    assert codes_a.shape[1] == code_words(d, enc) and codes_b.shape[1] == code_words(d, enc)
    assert ia.size == 0 or (ia.min() >= 0 and ia.max() < codes_a.shape[0])
    assert ib.size == 0 or (ib.min() >= 0 and ib.max() < codes_b.shape[0])
    out = np.zeros(ia.size, dtype=np.uint32)
    _check(_load().orc_distance_pairs_enc(_ptr(codes_a), _ptr(ia), _ptr(codes_b), _ptr(ib), ia.size, int(d), int(enc),
                                          _ptr(out)), "orc_distance_pairs_enc")
    return out


@dataclass
class SearchResult:
    ids: np.ndarray | None         # [nq, k] uint32, EMPTY padded
    scores: np.ndarray | None      # [nq, k] float32, -inf padded
    cand_ids: np.ndarray           # [nq, ef] uint32, sorted by (dist, id), EMPTY padded
    cand_dist: np.ndarray          # [nq, ef] uint32
    n_cand: np.ndarray             # [nq] uint32
    n_expanded: np.ndarray         # [nq] uint32
    n_dist_evals: np.ndarray       # [nq] uint32
    visit_order: np.ndarray | None  # [nq, visit_cap] uint32, EMPTY padded


def search(queries, adj, codes, vecs, entry: int, k: int, ef: int, visit_cap: int = 0,
           threads: int = 1, enc: int = SM) -> SearchResult:
    """Encode queries, beam-search the graph in code space, rerank with float32 cosine.

    vecs=None skips the rerank (ids/scores are None).
    """
    queries = _c(queries, np.float32)
    if queries.ndim == 1:
        queries = queries[None, :]
    adj = _c(adj, np.uint32)
    codes = _c(codes, np.uint64)
    nq, d = queries.shape
    n, R = adj.shape
    assert codes.shape == (n, code_words(d, enc))
    if vecs is not None:
        vecs = _c(vecs, np.float32)
        assert vecs.shape == (n, d)
    ids = np.zeros((nq, k), dtype=np.uint32) if vecs is not None else None
    scores = np.zeros((nq, k), dtype=np.float32) if vecs is not None else None
    cand_ids = np.zeros((nq, ef), dtype=np.uint32)
    cand_dist = np.zeros((nq, ef), dtype=np.uint32)
    counters = np.zeros((nq, 3), dtype=np.uint32)
    order = np.zeros((nq, visit_cap), dtype=np.uint32) if visit_cap > 0 else None
    rc = _load().orc_search_enc(int(enc), _ptr(queries), nq, n, d, R, _ptr(adj), _ptr(codes), _ptr(vecs), int(entry),
                                int(k), int(ef), _ptr(ids), _ptr(scores), _ptr(cand_ids), _ptr(cand_dist),
                                _ptr(counters), _ptr(order), int(visit_cap), int(threads))
    _check(rc, "orc_search_enc")
    return SearchResult(ids, scores, cand_ids, cand_dist, counters[:, 0].copy(), counters[:, 1].copy(),
                        counters[:, 2].copy(), order)


def rerank(queries, vecs, cand_ids, n_cand, k: int):
    """Cosine rerank of given candidate lists -> (ids [nq,k], scores [nq,k], all_scores [nq,ef])."""
    queries = _c(queries, np.float32)
    vecs = _c(vecs, np.float32)
    cand_ids = _c(cand_ids, np.uint32)
    n_cand = _c(n_cand, np.uint32)
    nq, d = queries.shape
    ef = cand_ids.shape[1]
    ids = np.zeros((nq, k), dtype=np.uint32)
    scores = np.zeros((nq, k), dtype=np.float32)
    all_scores = np.full((nq, ef), -np.inf, dtype=np.float32)
    _check(_load().orc_rerank(_ptr(queries), nq, d, _ptr(vecs), _ptr(cand_ids), ef, _ptr(n_cand), int(k),
                              _ptr(ids), _ptr(scores), _ptr(all_scores)), "orc_rerank")
    return ids, scores, all_scores


def bq_scan(codes, qcodes, d: int, K: int, threads: int = 1, enc: int = SM):
    """Brute force in code space: (ids [nq,K], dist [nq,K]) of the K smallest (distance, id) per query code."""
    codes = _c(codes, np.uint64)
    qcodes = _c(qcodes, np.uint64)
    assert codes.shape[1] == code_words(d, enc) and qcodes.shape[1] == code_words(d, enc)
    nq = qcodes.shape[0]
    ids = np.zeros((nq, K), dtype=np.uint32)
    dist = np.zeros((nq, K), dtype=np.uint32)
    _check(_load().orc_bq_scan_enc(int(enc), _ptr(codes), codes.shape[0], int(d), _ptr(qcodes), nq, int(K), _ptr(ids),
                                   _ptr(dist), int(threads)), "orc_bq_scan_enc")
    return ids, dist


def cosine_topk(vecs, queries, K: int, threads: int = 1):
    """Exact top-K by cosine on the float32 data (double accumulation) -> ids [nq,K]."""
    vecs = _c(vecs, np.float32)
    queries = _c(queries, np.float32)
    nq, d = queries.shape
    ids = np.zeros((nq, K), dtype=np.uint32)
    _check(_load().orc_cosine_topk(_ptr(vecs), vecs.shape[0], d, _ptr(queries), nq, int(K), _ptr(ids), int(threads)),
           "orc_cosine_topk")
    return ids


def topk_overlap(a, b) -> float:
    a = _c(a, np.uint32)
    b = _c(b, np.uint32)
    assert a.shape == b.shape
    return float(_load().orc_topk_overlap(_ptr(a), _ptr(b), a.shape[0], a.shape[1]))


def build_graph(codes, d: int, R: int, L: int, alpha: float, entry: int, max_batch: int = 1 << 20,
                enc: int = SM) -> np.ndarray:
    """Batch-synchronous construction in code space (Algorithm 1 + bidirectional re-selection) -> adj [n, R]."""
    codes = _c(codes, np.uint64)
    n = codes.shape[0]
    assert codes.shape[1] == code_words(d, enc)
    adj = np.zeros((n, R), dtype=np.uint32)
    _check(_load().orc_build_graph_enc(int(enc), _ptr(codes), n, int(d), int(R), int(L), float(alpha), int(entry),
                                       int(max_batch), _ptr(adj)), "orc_build_graph_enc")
    return adj
