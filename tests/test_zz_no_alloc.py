"""qv_search_static (the search entry point that allocates nothing: its scratch is a buffer inside the library's
device code) against qv_search, through the C ABI with raw ctypes: two calls in a row, the second smaller."""
import ctypes
import os

import numpy as np
import pytest
import torch

from tests import util
from workloads import datagen

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
P = ctypes.c_void_p
SCRATCH_BYTES = 16 << 20


class Trace(ctypes.Structure):
    _fields_ = [("cand_ids", P), ("cand_dist", P), ("n_cand", P), ("n_expanded", P), ("n_dist_evals", P),
                ("visit_order", P), ("visit_cap", ctypes.c_int64), ("status", P)]


@pytest.fixture(scope="module")
def lib():
    assert torch.cuda.is_available(), "these tests need the GPU"
    lib = ctypes.CDLL(os.path.join(ROOT, "paper_2605_02171_amd", "libquiver_hip.so"))
    lib.qv_encode.argtypes = [P, ctypes.c_int64, ctypes.c_int, P, P, P]
    lib.qv_index_load.argtypes = [ctypes.POINTER(P), ctypes.c_int64, ctypes.c_int, ctypes.c_int, P, P, P, ctypes.c_uint32]
    lib.qv_index_free.argtypes = [P]
    lib.qv_index_free.restype = None
    lib.qv_index_set_tuning.argtypes = [P] + [ctypes.c_int] * 5
    lib.qv_search_workspace_bytes.restype = ctypes.c_size_t
    lib.qv_search_workspace_bytes.argtypes = [ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int]
    lib.qv_search.argtypes = [P, P, ctypes.c_int64, ctypes.c_int, ctypes.c_int, P, P, P, ctypes.c_size_t,
                              ctypes.POINTER(Trace), P]
    lib.qv_search_static.argtypes = [P, P, ctypes.c_int64, ctypes.c_int, ctypes.c_int, P, P, ctypes.POINTER(Trace), P]
    return lib


def _outputs(nq, k, ef, cap):
    i32 = lambda *s: torch.full(s, 0x5A5A5A5A, dtype=torch.int32, device="cuda")
    t = dict(ids=i32(nq, k), scores=torch.full((nq, k), 7.0, dtype=torch.float32, device="cuda"), cand_ids=i32(nq, ef),
             cand_dist=i32(nq, ef), n_cand=i32(nq), n_expanded=i32(nq), n_dist_evals=i32(nq), visit_order=i32(nq, cap),
             status=i32(nq))
    tr = Trace(t["cand_ids"].data_ptr(), t["cand_dist"].data_ptr(), t["n_cand"].data_ptr(), t["n_expanded"].data_ptr(),
               t["n_dist_evals"].data_ptr(), t["visit_order"].data_ptr(), cap, t["status"].data_ptr())
    return t, tr


def _both(lib, index, q, k, ef, cap=200):
    nq, d = q.shape
    stream = torch.cuda.current_stream().cuda_stream
    want, tr_w = _outputs(nq, k, ef, cap)
    need = lib.qv_search_workspace_bytes(nq, d, k, ef)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    assert lib.qv_search(index, q.data_ptr(), nq, k, ef, want["ids"].data_ptr(), want["scores"].data_ptr(), ws.data_ptr(),
                         need, ctypes.byref(tr_w), stream) == 0
    got, tr_g = _outputs(nq, k, ef, cap)
    assert lib.qv_search_static(index, q.data_ptr(), nq, k, ef, got["ids"].data_ptr(), got["scores"].data_ptr(),
                                ctypes.byref(tr_g), stream) == 0
    torch.cuda.synchronize()
    for name in want:
        # the same kernels on the same inputs: integer outputs bit for bit, and the scores too
        assert torch.equal(got[name], want[name]), name
    return got


@pytest.mark.parametrize("d,R,rerank_mode", [(768, 64, 1), (384, 32, 2), (384, 32, 0), (768, 64, 3)])
def test_static_scratch_search_equals_workspace_search_twice_in_a_row(lib, d, R, rerank_mode):
    rng = np.random.default_rng(d)
    n = 20_000
    x = torch.from_numpy(rng.standard_normal((n, d)).astype(np.float32)).cuda()
    adj = torch.from_numpy(datagen.random_regular_graph(n, R, seed=d, fill=0.9).view(np.int32)).cuda()
    codes = torch.empty((n, 2 * ((d + 63) // 64)), dtype=torch.int64, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    assert lib.qv_encode(x.data_ptr(), n, d, codes.data_ptr(), None, stream) == 0
    index = P()
    assert lib.qv_index_load(ctypes.byref(index), n, d, R, adj.data_ptr(), codes.data_ptr(), x.data_ptr(), 3) == 0
    try:
        assert lib.qv_index_set_tuning(index, 0, 0, 0, 0, rerank_mode) == 0   # where Stage 2 runs: 0 = default
        big = torch.from_numpy(rng.standard_normal((5000, d)).astype(np.float32)).cuda()
        small = torch.from_numpy(rng.standard_normal((37, d)).astype(np.float32)).cuda()
        util.note(f"static scratch: d={d} first call, 5000 queries, ef=64")
        _both(lib, index, big, 10, 64)
        util.note(f"static scratch: d={d} second call, 37 queries, ef=100")
        _both(lib, index, small, 20, 100)
        util.note(f"static scratch: d={d} third call, 1 query, ef=1")
        _both(lib, index, small[:1].contiguous(), 1, 1)
        # a batch that does not fit the built-in buffer is refused before anything is launched
        nq_big = 200_000
        assert lib.qv_search_workspace_bytes(nq_big, d, 10, 64) > SCRATCH_BYTES
        rc = lib.qv_search_static(index, big.data_ptr(), nq_big, 10, 64, None, None, None, stream)
        assert rc in (-10, -2)
        ids = torch.empty((nq_big, 10), dtype=torch.int32, device="cuda")
        sc = torch.empty((nq_big, 10), dtype=torch.float32, device="cuda")
        assert lib.qv_search_static(index, big.data_ptr(), nq_big, 10, 64, ids.data_ptr(), sc.data_ptr(), None, stream) == -10
        assert lib.qv_search_static(index, big.data_ptr(), 10, 10, 5, ids.data_ptr(), sc.data_ptr(), None, stream) == -4
        torch.cuda.synchronize()
    finally:
        lib.qv_index_free(index)
