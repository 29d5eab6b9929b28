"""Thin ctypes binding of ``libquiver_hip.so`` (the C ABI declared in ``include/quiver.h``).

Argument marshalling only: torch tensors supply device memory and the current stream; every step
of the method runs in the library's HIP kernels.  There is no CPU fallback -- if the shared
library has not been built, importing this module raises.

Unsigned device arrays are carried in signed torch dtypes of the same width (codes: int64 holding
uint64 bit patterns; ids, distances, counters: int32 holding uint32).  ``to_numpy_u32`` /
``to_numpy_u64`` reinterpret them on the host.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libquiver_hip.so")

EMPTY = 0xFFFFFFFF
VISITED_EXACT = 1
VISITED_CACHE = 2
RERANK_SEPARATE = 1
RERANK_FUSED = 2
RERANK_TAIL = 3
ENC_SM, ENC_SIGN1, ENC_SQ2 = 0, 1, 2
STATUS_NONFINITE = 1
STATUS_VISITED_FULL = 2
STATUS_BAD_EDGE = 4
MAX_EF = 1024
STATIC_SCRATCH_BYTES = 16 << 20

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `python -m paper_2605_02171_amd.build` "
        "(hipcc, gfx950). There is no fallback path.")

_lib = ctypes.CDLL(LIB_PATH)
_P = ctypes.c_void_p


class _Trace(ctypes.Structure):
    _fields_ = [("cand_ids", _P), ("cand_dist", _P), ("n_cand", _P), ("n_expanded", _P), ("n_dist_evals", _P),
                ("visit_order", _P), ("visit_cap", ctypes.c_int64), ("status", _P)]


_lib.qv_code_words.restype = ctypes.c_int
_lib.qv_code_words.argtypes = [ctypes.c_int]
_lib.qv_encode.restype = ctypes.c_int
_lib.qv_encode.argtypes = [_P, ctypes.c_int64, ctypes.c_int, _P, _P, _P]
_lib.qv_bq_distance.restype = ctypes.c_int
_lib.qv_bq_distance.argtypes = [_P, _P, _P, _P, ctypes.c_int64, ctypes.c_int, _P, _P]
_lib.qv_gather_probe.restype = ctypes.c_int
_lib.qv_gather_probe.argtypes = [_P, ctypes.c_int64, ctypes.c_int, _P, ctypes.c_int64, _P, _P]
_lib.qv_bq_scan_workspace_bytes.restype = ctypes.c_size_t
_lib.qv_bq_scan_workspace_bytes.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int]
_lib.qv_bq_scan.restype = ctypes.c_int
_lib.qv_bq_scan.argtypes = [_P, ctypes.c_int64, ctypes.c_int, _P, ctypes.c_int64, ctypes.c_int, _P, _P, _P,
                            ctypes.c_size_t, _P]
_lib.qv_topk_overlap.restype = ctypes.c_int
_lib.qv_topk_overlap.argtypes = [_P, _P, ctypes.c_int64, ctypes.c_int, _P, _P]
_lib.qv_build_workspace_bytes.restype = ctypes.c_size_t
_lib.qv_build_workspace_bytes.argtypes = [ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int64]
_lib.qv_build_workspace_bytes_enc.restype = ctypes.c_size_t
_lib.qv_build_workspace_bytes_enc.argtypes = [ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int64]
_lib.qv_build_graph.restype = ctypes.c_int
_lib.qv_build_graph.argtypes = [_P, ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_double,
                                ctypes.c_uint32, ctypes.c_int64, _P, _P, ctypes.c_size_t, _P]
_lib.qv_index_load.restype = ctypes.c_int
_lib.qv_index_load.argtypes = [ctypes.POINTER(_P), ctypes.c_int64, ctypes.c_int, ctypes.c_int, _P, _P, _P,
                               ctypes.c_uint32]
_lib.qv_index_free.restype = None
_lib.qv_index_free.argtypes = [_P]
_lib.qv_index_set_tuning.restype = ctypes.c_int
_lib.qv_index_set_tuning.argtypes = [_P, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int]
_lib.qv_code_words_enc.restype = ctypes.c_int
_lib.qv_code_words_enc.argtypes = [ctypes.c_int, ctypes.c_int]
_lib.qv_encode_enc.restype = ctypes.c_int
_lib.qv_encode_enc.argtypes = [_P, ctypes.c_int64, ctypes.c_int, ctypes.c_int, _P, _P, _P]
_lib.qv_bq_distance_enc.restype = ctypes.c_int
_lib.qv_bq_distance_enc.argtypes = [_P, _P, _P, _P, ctypes.c_int64, ctypes.c_int, ctypes.c_int, _P, _P]
_lib.qv_bq_scan_enc.restype = ctypes.c_int
_lib.qv_bq_scan_enc.argtypes = [_P, ctypes.c_int64, ctypes.c_int, ctypes.c_int, _P, ctypes.c_int64, ctypes.c_int, _P, _P, _P,
                                ctypes.c_size_t, _P]
_lib.qv_build_graph_enc.restype = ctypes.c_int
_lib.qv_build_graph_enc.argtypes = [_P, ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                    ctypes.c_double, ctypes.c_uint32, ctypes.c_int64, _P, _P, ctypes.c_size_t, _P]
_lib.qv_index_set_encoding.restype = ctypes.c_int
_lib.qv_index_set_encoding.argtypes = [_P, ctypes.c_int]
_lib.qv_index_rerank_fused.restype = ctypes.c_int
_lib.qv_index_rerank_fused.argtypes = [_P, ctypes.c_int]
_lib.qv_code_layout.restype = ctypes.c_int
_lib.qv_code_layout.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int)]
_lib.qv_pad_codes.restype = ctypes.c_int
_lib.qv_pad_codes.argtypes = [_P, ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, _P, _P]
_lib.qv_index_set_code_layout.restype = ctypes.c_int
_lib.qv_index_set_code_layout.argtypes = [_P, ctypes.c_int, ctypes.c_int]
_lib.qv_split_layout.restype = ctypes.c_int
_lib.qv_split_layout.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int)]
_lib.qv_split_codes.restype = ctypes.c_int
_lib.qv_split_codes.argtypes = [_P, ctypes.c_int64, ctypes.c_int, _P, _P, _P]
_lib.qv_index_set_split_codes.restype = ctypes.c_int
_lib.qv_index_set_split_codes.argtypes = [_P, _P, _P]
_lib.qv_search_workspace_bytes.restype = ctypes.c_size_t
_lib.qv_search_workspace_bytes.argtypes = [ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int]
_lib.qv_search.restype = ctypes.c_int
_lib.qv_search.argtypes = [_P, _P, ctypes.c_int64, ctypes.c_int, ctypes.c_int, _P, _P, _P, ctypes.c_size_t,
                           ctypes.POINTER(_Trace), _P]
_lib.qv_search_static.restype = ctypes.c_int
_lib.qv_search_static.argtypes = [_P, _P, ctypes.c_int64, ctypes.c_int, ctypes.c_int, _P, _P, ctypes.POINTER(_Trace), _P]
_lib.qv_timer_create.restype = ctypes.c_int
_lib.qv_timer_create.argtypes = [ctypes.POINTER(_P), ctypes.c_int]
_lib.qv_timer_free.restype = None
_lib.qv_timer_free.argtypes = [_P]
_lib.qv_index_set_timer.restype = None
_lib.qv_index_set_timer.argtypes = [_P, _P]
_lib.qv_timer_read.restype = ctypes.c_int
_lib.qv_timer_read.argtypes = [_P, _P, ctypes.c_int]
_lib.qv_strerror.restype = ctypes.c_char_p
_lib.qv_strerror.argtypes = [ctypes.c_int]
_lib.qv_last_hip_error.restype = ctypes.c_char_p
_lib.qv_last_hip_error.argtypes = []


class QuiverError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        msg = _lib.qv_strerror(code).decode()
        hip = _lib.qv_last_hip_error().decode()
        super().__init__(f"{what}: {msg} ({code})" + (f" [{hip}]" if code == -7 and hip else ""))


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise QuiverError(rc, what)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dev(t: torch.Tensor, dtype: torch.dtype, what: str) -> torch.Tensor:
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{what} must be a CUDA/HIP torch tensor")
    if t.dtype != dtype or not t.is_contiguous():
        raise TypeError(f"{what} must be contiguous {dtype}, got {t.dtype}")
    return t


def to_numpy_u32(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().numpy().view(np.uint32)


def to_numpy_u64(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().numpy().view(np.uint64)


def from_numpy_u32(a: np.ndarray, device="cuda") -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint32).view(np.int32)).to(device)


def from_numpy_u64(a: np.ndarray, device="cuda") -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint64).view(np.int64)).to(device)


def code_words(d: int, enc: int = ENC_SM) -> int:
    return _lib.qv_code_words_enc(int(d), int(enc))


def encode(x: torch.Tensor, want_status: bool = False, enc: int = ENC_SM):
    """qv_encode / qv_encode_enc: float32 [n, d] on the device -> int64 [n, code_words(d, enc)] (uint64 bit patterns)."""
    x = _dev(x, torch.float32, "x")
    if x.dim() != 2:
        raise ValueError("x must be [n, d]")
    n, d = x.shape
    cw = code_words(d, enc)
    if cw == 0:
        raise QuiverError(-3 if enc in (ENC_SM, ENC_SIGN1, ENC_SQ2) else -1, "qv_encode")
    codes = torch.empty((n, cw), dtype=torch.int64, device=x.device)
    status = torch.empty((n,), dtype=torch.int32, device=x.device) if want_status else None
    _check(_lib.qv_encode_enc(x.data_ptr(), n, d, int(enc), codes.data_ptr(),
                              status.data_ptr() if want_status else None, _stream()), "qv_encode_enc")
    return (codes, status) if want_status else codes


def code_layout(d: int, enc: int = ENC_SM) -> tuple[int, int]:
    """qv_code_layout: (plane_words, stride) recommended for an index's codes (compiled plane width, line-aligned rows)."""
    pw, st = ctypes.c_int(0), ctypes.c_int(0)
    _check(_lib.qv_code_layout(int(d), int(enc), ctypes.byref(pw), ctypes.byref(st)), "qv_code_layout")
    return pw.value, st.value


def pad_codes(codes: torch.Tensor, d: int, layout: tuple[int, int] | None = None, enc: int = ENC_SM) -> torch.Tensor:
    """qv_pad_codes: dense [n, cw] code rows -> [n, stride] rows in `layout` = (plane_words, stride); default: code_layout."""
    codes = _dev(codes, torch.int64, "codes")
    if codes.dim() != 2 or codes.shape[1] != code_words(d, enc):
        raise ValueError("codes must be [n, code_words(d)]")
    pw, stride = code_layout(d, enc) if layout is None else (int(layout[0]), int(layout[1]))
    out = torch.empty((codes.shape[0], stride), dtype=torch.int64, device=codes.device)
    _check(_lib.qv_pad_codes(codes.data_ptr(), codes.shape[0], d, int(enc), pw, stride, out.data_ptr(), _stream()),
           "qv_pad_codes")
    return out


def split_layout(d: int) -> tuple[int, int] | None:
    """qv_split_layout: row lengths (64-bit words) of the two arrays of the split layout, or None where it does not apply."""
    w1, w2 = ctypes.c_int(0), ctypes.c_int(0)
    rc = _lib.qv_split_layout(int(d), ctypes.byref(w1), ctypes.byref(w2))
    if rc == -9:
        return None
    _check(rc, "qv_split_layout")
    return w1.value, w2.value


def split_codes(codes: torch.Tensor, d: int) -> tuple[torch.Tensor, torch.Tensor]:
    """qv_split_codes: dense Sign-Magnitude rows [n, cw] -> ([n, words1], [n, words2]) in the split layout."""
    codes = _dev(codes, torch.int64, "codes")
    if codes.dim() != 2 or codes.shape[1] != code_words(d):
        raise ValueError("codes must be [n, code_words(d)]")
    lay = split_layout(d)
    if lay is None:
        raise QuiverError(-9, "qv_split_layout")
    n = codes.shape[0]
    out1 = torch.empty((n, lay[0]), dtype=torch.int64, device=codes.device)
    out2 = torch.empty((n, lay[1]), dtype=torch.int64, device=codes.device)
    _check(_lib.qv_split_codes(codes.data_ptr(), n, int(d), out1.data_ptr(), out2.data_ptr(), _stream()), "qv_split_codes")
    return out1, out2


def bq_distance(codes_a: torch.Tensor, ia: torch.Tensor, codes_b: torch.Tensor, ib: torch.Tensor, d: int,
                enc: int = ENC_SM):
    """qv_bq_distance(_enc): code distance for index pairs -> int32 [npairs] (uint32 values)."""
    codes_a = _dev(codes_a, torch.int64, "codes_a")
    codes_b = _dev(codes_b, torch.int64, "codes_b")
    ia = _dev(ia, torch.int64, "ia")
    ib = _dev(ib, torch.int64, "ib")
    cw = code_words(d, enc)
    if codes_a.shape[1] != cw or codes_b.shape[1] != cw or ia.shape != ib.shape:
        raise ValueError("shape mismatch")
    if ia.numel() and (int(ia.min()) < 0 or int(ia.max()) >= codes_a.shape[0] or int(ib.min()) < 0 or
                       int(ib.max()) >= codes_b.shape[0]):
        raise IndexError("pair index out of range")
    out = torch.empty(ia.shape, dtype=torch.int32, device=codes_a.device)
    _check(_lib.qv_bq_distance_enc(codes_a.data_ptr(), ia.data_ptr(), codes_b.data_ptr(), ib.data_ptr(), ia.numel(),
                                   int(d), int(enc), out.data_ptr(), _stream()), "qv_bq_distance_enc")
    return out


def gather_probe(codes: torch.Tensor, d: int, ids: torch.Tensor) -> None:
    """qv_gather_probe: read the code rows named by ids (int32 holding uint32, all < n) and discard them."""
    codes = _dev(codes, torch.int64, "codes")
    ids = _dev(ids, torch.int32, "ids")
    sink = torch.zeros(1, dtype=torch.int64, device=codes.device)
    _check(_lib.qv_gather_probe(codes.data_ptr(), codes.shape[0], int(d), ids.data_ptr(), ids.numel(),
                                sink.data_ptr(), _stream()), "qv_gather_probe")


def bq_scan(codes: torch.Tensor, qcodes: torch.Tensor, d: int, K: int, enc: int = ENC_SM):
    """qv_bq_scan(_enc): brute force in code space -> (ids, dist) int32 [nq, K] holding uint32 values."""
    codes = _dev(codes, torch.int64, "codes")
    qcodes = _dev(qcodes, torch.int64, "qcodes")
    cw = code_words(d, enc)
    if codes.shape[1] != cw or qcodes.shape[1] != cw:
        raise ValueError("code width does not match d")
    n, nq = codes.shape[0], qcodes.shape[0]
    ids = torch.empty((nq, K), dtype=torch.int32, device=codes.device)
    dist = torch.empty((nq, K), dtype=torch.int32, device=codes.device)
    need = int(_lib.qv_bq_scan_workspace_bytes(n, nq, K))
    ws = torch.empty((max(need, 256),), dtype=torch.uint8, device=codes.device)
    _check(_lib.qv_bq_scan_enc(codes.data_ptr(), n, int(d), int(enc), qcodes.data_ptr(), nq, int(K), ids.data_ptr(),
                               dist.data_ptr(), ws.data_ptr(), ws.numel(), _stream()), "qv_bq_scan_enc")
    return ids, dist


def topk_overlap(a: torch.Tensor, b: torch.Tensor) -> torch.Tensor:
    """qv_topk_overlap: per-query count of ids of a[q] that occur in b[q] (int32 [nq])."""
    a = _dev(a, torch.int32, "a")
    b = _dev(b, torch.int32, "b")
    if a.shape != b.shape or a.dim() != 2:
        raise ValueError("a and b must both be [nq, K]")
    hits = torch.empty((a.shape[0],), dtype=torch.int32, device=a.device)
    _check(_lib.qv_topk_overlap(a.data_ptr(), b.data_ptr(), a.shape[0], a.shape[1], hits.data_ptr(), _stream()),
           "qv_topk_overlap")
    return hits


def build_graph(codes: torch.Tensor, d: int, R: int, L: int, alpha: float, entry: int,
                max_batch: int = 1 << 20, enc: int = ENC_SM) -> torch.Tensor:
    """qv_build_graph(_enc): batch-synchronous construction in code space -> adj int32 [n, R] (uint32 bits)."""
    codes = _dev(codes, torch.int64, "codes")
    n = codes.shape[0]
    if codes.shape[1] != code_words(d, enc):
        raise ValueError("code width does not match d")
    need = int(_lib.qv_build_workspace_bytes_enc(n, int(d), int(enc), int(R), int(L), int(max_batch)))
    ws = torch.empty((max(need, 256),), dtype=torch.uint8, device=codes.device)
    adj = torch.empty((n, R), dtype=torch.int32, device=codes.device)
    _check(_lib.qv_build_graph_enc(codes.data_ptr(), n, int(d), int(enc), int(R), int(L), float(alpha), int(entry),
                                   int(max_batch), adj.data_ptr(), ws.data_ptr(), ws.numel(), _stream()),
           "qv_build_graph_enc")
    return adj


class Timer:
    """qv_timer: per-stage HIP-event timing of the searches of one index."""

    def __init__(self, max_calls: int):
        self.max_calls = max_calls
        h = _P()
        _check(_lib.qv_timer_create(ctypes.byref(h), max_calls), "qv_timer_create")
        self._h = h

    def read(self) -> np.ndarray:
        """Milliseconds [calls, 3] = (query encode + launch-order pass, beam search kernel, rerank); waits for the events."""
        ms = np.zeros((self.max_calls, 3), dtype=np.float32)
        n = _lib.qv_timer_read(self._h, ms.ctypes.data_as(_P), self.max_calls)
        if n < 0:
            raise QuiverError(n, "qv_timer_read")
        return ms[:n]

    def __del__(self):
        if getattr(self, "_h", None):
            _lib.qv_timer_free(self._h)
            self._h = None


class Index:
    """qv_index_load: borrows adj [n, R] (int32/uint32 bits), codes [n, cw] int64, vecs [n, d] float32.

    With ``layout=(plane_words, stride)`` codes is [n, stride] as ``pad_codes`` wrote it.

    vecs may be a device tensor or a pinned host tensor (``pin_memory=True``): the float32 vectors are the
    cold data of the method and are only touched by the rerank.
    """

    def __init__(self, adj: torch.Tensor, codes: torch.Tensor, vecs: torch.Tensor, entry: int, enc: int = ENC_SM,
                 layout: tuple[int, int] | None = None):
        adj = _dev(adj, torch.int32, "adj")
        codes = _dev(codes, torch.int64, "codes")
        if isinstance(vecs, torch.Tensor) and not vecs.is_cuda and vecs.is_pinned():
            # cold store kept in pinned host memory: the device addresses it directly, only the rerank reads it
            if vecs.dtype != torch.float32 or not vecs.is_contiguous():
                raise TypeError("vecs must be contiguous float32")
        else:
            vecs = _dev(vecs, torch.float32, "vecs")
        n, d = vecs.shape
        row = code_words(d, enc) if layout is None else int(layout[1])
        if adj.shape[0] != n or codes.shape != (n, row):
            raise ValueError("adj/codes/vecs shapes do not agree")
        self.n, self.d, self.R = n, d, adj.shape[1]
        self._keep = (adj, codes, vecs)  # the library borrows these buffers
        h = _P()
        _check(_lib.qv_index_load(ctypes.byref(h), n, d, self.R, adj.data_ptr(), codes.data_ptr(), vecs.data_ptr(),
                                  int(entry)), "qv_index_load")
        self._h = h
        self._timer = None
        if enc != ENC_SM:
            _check(_lib.qv_index_set_encoding(h, int(enc)), "qv_index_set_encoding")
        if layout is not None:
            _check(_lib.qv_index_set_code_layout(h, int(layout[0]), int(layout[1])), "qv_index_set_code_layout")

    def set_split_codes(self, split: tuple[torch.Tensor, torch.Tensor] | None) -> None:
        """qv_index_set_split_codes: the index's codes in the split layout as well (None: forget them)."""
        if split is None:
            _check(_lib.qv_index_set_split_codes(self._h, None, None), "qv_index_set_split_codes")
            self._split = None
            return
        a, b = _dev(split[0], torch.int64, "split[0]"), _dev(split[1], torch.int64, "split[1]")
        lay = split_layout(self.d)
        if lay is None or a.shape != (self.n, lay[0]) or b.shape != (self.n, lay[1]):
            raise ValueError("split arrays do not match the index")
        _check(_lib.qv_index_set_split_codes(self._h, a.data_ptr(), b.data_ptr()), "qv_index_set_split_codes")
        self._split = (a, b)

    def set_tuning(self, visited_slots: int = 0, lanes_per_row: int = 0, table_format: int = 0,
                   visited_mode: int = 0, rerank_mode: int = 0) -> None:
        _check(_lib.qv_index_set_tuning(self._h, visited_slots, lanes_per_row, table_format, visited_mode, rerank_mode),
               "qv_index_set_tuning")

    def rerank_fused(self, ef: int) -> bool:
        """qv_index_rerank_fused: does a search with this beam width score its lists inside the search kernel?"""
        return bool(_lib.qv_index_rerank_fused(self._h, int(ef)))

    def set_timer(self, timer: Timer | None) -> None:
        self._timer = timer
        _lib.qv_index_set_timer(self._h, timer._h if timer else None)

    def __del__(self):
        if getattr(self, "_h", None):
            _lib.qv_index_free(self._h)
            self._h = None


@dataclass
class SearchOutput:
    ids: torch.Tensor                 # [nq, k] int32 (uint32 bits), EMPTY padded
    scores: torch.Tensor              # [nq, k] float32
    cand_ids: torch.Tensor | None = None      # [nq, ef]
    cand_dist: torch.Tensor | None = None     # [nq, ef]
    n_cand: torch.Tensor | None = None        # [nq]
    n_expanded: torch.Tensor | None = None
    n_dist_evals: torch.Tensor | None = None
    visit_order: torch.Tensor | None = None   # [nq, visit_cap]
    status: torch.Tensor | None = None


def search_workspace_bytes(nq: int, d: int, k: int, ef: int) -> int:
    return int(_lib.qv_search_workspace_bytes(nq, d, k, ef))


def search(index: Index, queries: torch.Tensor, k: int, ef: int, trace: bool = False, visit_cap: int = 0,
           workspace: torch.Tensor | None = None, out: SearchOutput | None = None) -> SearchOutput:
    """qv_search: encode queries, beam search in code space, float32 cosine rerank -> top-k."""
    queries = _dev(queries, torch.float32, "queries")
    if queries.dim() != 2 or queries.shape[1] != index.d:
        raise ValueError("queries must be [nq, d]")
    nq = queries.shape[0]
    dev = queries.device
    need = search_workspace_bytes(nq, index.d, k, ef)
    if workspace is None and need > 0:
        workspace = torch.empty((need,), dtype=torch.uint8, device=dev)
    if out is None:
        i32 = lambda *s: torch.empty(s, dtype=torch.int32, device=dev)
        out = SearchOutput(i32(nq, k), torch.empty((nq, k), dtype=torch.float32, device=dev))
        if trace:
            out.cand_ids, out.cand_dist = i32(nq, max(ef, 0)), i32(nq, max(ef, 0))
            out.n_cand, out.n_expanded, out.n_dist_evals, out.status = i32(nq), i32(nq), i32(nq), i32(nq)
            if visit_cap > 0:
                out.visit_order = i32(nq, visit_cap)
    tr = None
    if out.cand_ids is not None or out.n_expanded is not None or out.visit_order is not None:
        ptr = lambda t: t.data_ptr() if t is not None else None
        tr = _Trace(ptr(out.cand_ids), ptr(out.cand_dist), ptr(out.n_cand), ptr(out.n_expanded),
                    ptr(out.n_dist_evals), ptr(out.visit_order),
                    out.visit_order.shape[1] if out.visit_order is not None else 0, ptr(out.status))
    rc = _lib.qv_search(index._h, queries.data_ptr(), nq, int(k), int(ef), out.ids.data_ptr(),
                        out.scores.data_ptr(), workspace.data_ptr() if workspace is not None else None,
                        workspace.numel() if workspace is not None else 0,
                        ctypes.byref(tr) if tr is not None else None, _stream())
    _check(rc, "qv_search")
    return out


def search_static(index: Index, queries: torch.Tensor, k: int, ef: int, out: SearchOutput) -> SearchOutput:
    """qv_search_static: qv_search on the library's built-in scratch buffer.  Every output tensor comes from the
    caller (``out``: ids and scores, plus whichever trace tensors are wanted), so the call allocates nothing."""
    queries = _dev(queries, torch.float32, "queries")
    if queries.dim() != 2 or queries.shape[1] != index.d:
        raise ValueError("queries must be [nq, d]")
    tr = None
    if out.cand_ids is not None or out.n_expanded is not None or out.visit_order is not None:
        ptr = lambda t: t.data_ptr() if t is not None else None
        tr = _Trace(ptr(out.cand_ids), ptr(out.cand_dist), ptr(out.n_cand), ptr(out.n_expanded),
                    ptr(out.n_dist_evals), ptr(out.visit_order),
                    out.visit_order.shape[1] if out.visit_order is not None else 0, ptr(out.status))
    rc = _lib.qv_search_static(index._h, queries.data_ptr(), queries.shape[0], int(k), int(ef), out.ids.data_ptr(),
                               out.scores.data_ptr(), ctypes.byref(tr) if tr is not None else None, _stream())
    _check(rc, "qv_search_static")
    return out
