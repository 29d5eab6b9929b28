"""The C-ABI library loads without a GPU, exports every function include/quiver.h declares, and rejects
bad arguments on the host before touching the device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "quiver.h")
LIB = os.path.join(ROOT, "paper_2605_02171_amd", "libquiver_hip.so")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2605_02171_amd import build
        build.build(force=True)
    return ctypes.CDLL(LIB)


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(qv_[a-z0-9_]+)\s*\(", text))
    assert len(names) >= 12
    return sorted(names)


def test_every_declared_function_is_exported(lib):
    for name in _declared_functions():
        assert hasattr(lib, name), f"{name} is declared in quiver.h but not exported"


def test_header_documents_each_entry_point():
    text = open(HEADER).read()
    for name in ("qv_encode", "qv_bq_distance", "qv_index_load", "qv_search"):
        head = text[:text.index(f"int {name}(")]
        comment = head[head.rindex("/*"):]
        assert "paper Sec." in comment, f"{name} does not cite the passage that defines it"


def test_sizes(lib):
    lib.qv_code_words.restype = ctypes.c_int
    assert [lib.qv_code_words(d) for d in (0, 1, 64, 65, 384, 768, 3072, 65536, 65537)] == \
        [0, 2, 2, 4, 12, 24, 96, 2048, 0]
    f = lib.qv_search_workspace_bytes
    f.restype = ctypes.c_size_t
    f.argtypes = [ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int]
    assert f(10, 768, 10, 64) >= 10 * (24 * 8 + 64 * 8 + 4)
    assert f(10, 768, 65, 64) == 0 and f(10, 0, 1, 8) == 0 and f(10, 768, 1, 2000) == 0 and f(-1, 8, 1, 8) == 0


def test_line_aligned_row_strides(lib):
    """The recommended stride is the dense row unless padding lowers the mean number of 128-byte lines a row
    touches; check that against a brute-force count over every row offset."""
    f = lib.qv_code_stride_words
    f.restype = ctypes.c_int
    f.argtypes = [ctypes.c_int, ctypes.c_int]
    g = lib.qv_code_words_enc
    g.restype = ctypes.c_int
    g.argtypes = [ctypes.c_int, ctypes.c_int]

    def mean_lines(row_bytes, stride_bytes):
        total = 0
        for i in range(128):                      # offsets repeat after at most 128 rows
            a = i * stride_bytes
            total += (a + row_bytes - 1) // 128 - a // 128 + 1
        return total / 128

    assert [f(d, 0) for d in (64, 128, 192, 384, 512, 768, 960, 1024, 3072)] == [2, 4, 8, 16, 16, 24, 32, 32, 96]
    assert [f(d, 1) for d in (64, 192, 384, 768, 960)] == [1, 4, 8, 16, 16]
    assert f(0, 0) == 0 and f(768, 9) == 0 and f(70000, 0) == 0
    for enc in (0, 1, 2):
        for d in list(range(1, 2200, 37)) + [64, 384, 768, 960, 1024, 1536, 3072, 65536]:
            words, stride = g(d, enc), f(d, enc)
            assert stride >= words and (stride == words or stride % 2 == 0) and stride <= 4 * words + 16
            dense, chosen = mean_lines(words * 8, words * 8), mean_lines(words * 8, stride * 8)
            assert chosen <= dense
            if stride != words:
                assert chosen < dense                                      # padding only when it pays
                assert chosen == max(1, -(-words * 8 // 128))             # and then a row touches the fewest lines possible
            else:                                                          # no aligned stride would do better
                bytes_ = words * 8
                aligned = next(s for s in (16, 32, 64) if s >= bytes_) if bytes_ <= 64 else -(-bytes_ // 128) * 128
                assert mean_lines(bytes_, aligned) >= dense


def test_host_side_argument_errors(lib):
    P = ctypes.c_void_p
    fake = P(0x1000)  # never dereferenced: every call below fails before any launch
    lib.qv_encode.argtypes = [P, ctypes.c_int64, ctypes.c_int, P, P, P]
    assert lib.qv_encode(fake, 4, 0, fake, None, None) == -3
    assert lib.qv_encode(fake, 4, 70000, fake, None, None) == -3
    assert lib.qv_encode(None, 4, 8, fake, None, None) == -2
    assert lib.qv_encode(fake, -1, 8, fake, None, None) == -1
    assert lib.qv_encode(fake, (1 << 32) + 1, 8, fake, None, None) == -1
    assert lib.qv_encode(None, 0, 8, None, None, None) == 0          # empty input is fine
    lib.qv_bq_distance.argtypes = [P, P, P, P, ctypes.c_int64, ctypes.c_int, P, P]
    assert lib.qv_bq_distance(fake, fake, fake, None, 3, 8, fake, None) == -2
    assert lib.qv_bq_distance(fake, fake, fake, fake, 3, 0, fake, None) == -3
    lib.qv_index_load.argtypes = [ctypes.POINTER(P), ctypes.c_int64, ctypes.c_int, ctypes.c_int, P, P, P, ctypes.c_uint32]
    h = P()
    assert lib.qv_index_load(ctypes.byref(h), 10, 8, 4, fake, fake, fake, 10) == -1   # entry out of range
    assert lib.qv_index_load(ctypes.byref(h), 10, 8, 0, fake, fake, fake, 0) == -1    # R < 1
    assert lib.qv_index_load(ctypes.byref(h), 10, 8, 4, None, fake, fake, 0) == -2
    assert lib.qv_index_load(ctypes.byref(h), 10, 0, 4, fake, fake, fake, 0) == -3
    assert lib.qv_index_load(None, 10, 8, 4, fake, fake, fake, 0) == -2
    assert lib.qv_index_load(ctypes.byref(h), 10, 8, 4, fake, fake, fake, 3) == 0 and h.value
    lib.qv_search.argtypes = [P, P, ctypes.c_int64, ctypes.c_int, ctypes.c_int, P, P, P, ctypes.c_size_t, P, P]
    assert lib.qv_search(None, fake, 1, 1, 8, fake, fake, fake, 1 << 20, None, None) == -2
    assert lib.qv_search(h, fake, 1, 9, 8, fake, fake, fake, 1 << 20, None, None) == -4
    assert lib.qv_search(h, fake, 1, 1, 0, fake, fake, fake, 1 << 20, None, None) == -5
    assert lib.qv_search(h, fake, 1, 1, 5000, fake, fake, fake, 1 << 20, None, None) == -5
    assert lib.qv_search(h, fake, 1, 1, 8, fake, fake, None, 0, None, None) == -6
    assert lib.qv_search(h, fake, 1, 1, 8, fake, fake, P(0x1001), 1 << 20, None, None) == -6   # misaligned
    assert lib.qv_search(h, fake, 1, 1, 8, fake, fake, fake, 16, None, None) == -6             # too small
    assert lib.qv_search(h, None, 1, 1, 8, fake, fake, fake, 1 << 20, None, None) == -2
    assert lib.qv_search(h, None, 0, 1, 8, None, None, None, 0, None, None) == 0               # empty batch
    lib.qv_index_set_tuning.argtypes = [P, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int]
    assert lib.qv_index_set_tuning(h, 512, 0, 0, 0) == -1 and lib.qv_index_set_tuning(h, 0, 3, 0, 0) == -1
    assert lib.qv_index_set_tuning(h, 0, 0, 16, 0) == -1 and lib.qv_index_set_tuning(h, 8192, 4, 32, 0) == 0
    assert lib.qv_index_set_tuning(h, 0, 0, 0, 3) == -1 and lib.qv_index_set_tuning(h, 4096, 2, 0, 2) == 0
    # row stride of the index's codes: the dense length, or even and longer (d = 8: one word per plane, 2 per row)
    lib.qv_index_set_code_stride.argtypes = [P, ctypes.c_int]
    assert lib.qv_index_set_code_stride(h, 0) == 0 and lib.qv_index_set_code_stride(h, 2) == 0
    assert lib.qv_index_set_code_stride(h, 4) == 0 and lib.qv_index_set_code_stride(h, 16) == 0
    assert lib.qv_index_set_code_stride(h, 1) == -1 and lib.qv_index_set_code_stride(h, 3) == -1
    assert lib.qv_index_set_code_stride(h, 4096) == -1 and lib.qv_index_set_code_stride(None, 2) == -2
    lib.qv_pad_codes.argtypes = [P, ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int, P, P]
    assert lib.qv_pad_codes(fake, 5, 384, 0, 11, fake, None) == -1       # shorter than the row
    assert lib.qv_pad_codes(fake, 5, 384, 0, 13, fake, None) == -1       # odd
    assert lib.qv_pad_codes(fake, 5, 384, 7, 16, fake, None) == -1       # unknown encoding
    assert lib.qv_pad_codes(fake, 5, 0, 0, 16, fake, None) == -3
    assert lib.qv_pad_codes(None, 5, 384, 0, 16, fake, None) == -2
    assert lib.qv_pad_codes(None, 0, 384, 0, 16, None, None) == 0        # nothing to do
    lib.qv_index_free.argtypes = [P]
    lib.qv_index_free(h)
    lib.qv_index_free(None)
    lib.qv_strerror.restype = ctypes.c_char_p
    assert b"ef" in lib.qv_strerror(-4) and lib.qv_strerror(0) == b"ok"


def test_workload_generators_are_deterministic_and_shaped():
    import numpy as np
    from workloads import datagen, graph
    w = datagen.scaled("C2", n=3000, nq=20)
    x1, x2 = datagen.make_base(w), datagen.make_base(w)
    assert (x1 == x2).all() and x1.shape == (3000, 768) and x1.dtype == np.float32
    np.testing.assert_allclose(np.linalg.norm(x1, axis=1), 1.0, atol=1e-5)
    sizes = datagen._cluster_sizes(1_000_000, 1024, 1.5)
    assert sizes.sum() == 1_000_000 and sizes.min() >= 1 and sizes[0] > sizes[10] > sizes[1000]
    g = datagen.make_base(datagen.scaled("C5", n=2000, nq=5))
    assert abs(float(g.std()) - 1.0) < 0.01
    a1, e1 = graph.build_graph(x1, 16, 24, 1.2, threads=1)
    a2, e2 = graph.build_graph(x1, 16, 24, 1.2, threads=4)
    assert e1 == e2 and (a1 == a2).all()                      # independent of the thread count
    deg = (a1 != 0xFFFFFFFF).sum(1)
    assert deg.max() <= 16 and (a1[a1 != 0xFFFFFFFF] < 3000).all()
    assert all(u not in row for u, row in enumerate(a1.tolist()))          # no self loops
    assert all(len(set(r) - {0xFFFFFFFF}) == (np.array(r) != 0xFFFFFFFF).sum() for r in a1.tolist())  # no duplicates


def test_graph_generator_entry_point_and_reachability_checked_with_the_oracle():
    # the generator has its own quick encoder and popcount distance; check what it derived from them
    # with the oracle's encoder and distance
    import numpy as np
    import oracle
    from tests import pyref
    from workloads import datagen, graph
    w = datagen.scaled("C1", n=1500, nq=5)
    x = datagen.make_base(w)
    adj, entry = graph.build_graph(x, 12, 32, 1.2, threads=2)
    codes = oracle.encode(x)
    centroid = x.astype(np.float64).mean(axis=0).astype(np.float32)
    cc = oracle.encode(centroid[None, :])
    d = oracle.sm_distance_pairs(cc, np.zeros(1500, dtype=np.int64), codes, np.arange(1500), w.d)
    assert entry == int(np.lexsort((np.arange(1500), d))[0])      # nearest code to the centroid's code, smallest id
    assert len(pyref.bfs_reachable(adj, entry)) >= 0.99 * 1500     # the graph is navigable from there
    # out-edges of a node that was never re-selected are sorted by (distance, id) as Algorithm 1 emits them;
    # at least the first edge of every non-empty row is the nearest of that row
    for t in range(0, 1500, 50):
        nb = [int(v) for v in adj[t] if v != 0xFFFFFFFF]
        assert nb and t not in nb
