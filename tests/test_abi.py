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


def _compiled_widths():
    """Plane widths the Sign-Magnitude search kernel is compiled for, from the source's own list."""
    src = open(os.path.join(ROOT, "paper_2605_02171_amd", "csrc", "search.hip")).read()
    line = re.search(r"#define QV_SM_WIDTHS\(X\)(.*)", src).group(1)
    return sorted(int(w) for w in re.findall(r"X\((\d+)\)", line))


def test_build_script_compiles_every_width_the_dispatcher_names():
    from paper_2605_02171_amd import build
    sm = sorted(w for e, w in build.SEARCH_VARIANTS if e == 0 and w != 0)
    assert sm == _compiled_widths()
    for e in (1, 2):
        assert sorted(w for enc, w in build.SEARCH_VARIANTS if enc == e and w != 0) == sm
    assert {(0, 0), (1, 0), (2, 0)} <= set(build.SEARCH_VARIANTS)


def test_recommended_code_layout(lib):
    """Planes go to the next compiled width when that costs at most a third more; the stride is the row unless
    padding lowers the mean number of 128-byte lines a row touches (checked by counting over every row offset)."""
    f = lib.qv_code_layout
    f.restype = ctypes.c_int
    f.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int)]

    def layout(d, enc):
        pw, st = ctypes.c_int(-1), ctypes.c_int(-1)
        assert f(d, enc, ctypes.byref(pw), ctypes.byref(st)) == 0
        return pw.value, st.value

    def mean_lines(row_bytes, stride_bytes):
        total = 0
        for i in range(128):                      # offsets repeat after at most 128 rows
            a = i * stride_bytes
            total += (a + row_bytes - 1) // 128 - a // 128 + 1
        return total / 128

    assert [layout(d, 0) for d in (64, 128, 192, 300, 384, 448, 512, 768, 960, 1024, 1100, 1536, 2048, 3072, 4096)] == \
        [(1, 2), (2, 4), (4, 8), (6, 16), (6, 16), (8, 16), (8, 16), (12, 24), (16, 32), (16, 32), (24, 48), (24, 48),
         (32, 64), (48, 96), (64, 128)]
    assert [layout(d, 1) for d in (64, 192, 384, 700, 768, 960)] == [(1, 1), (4, 4), (6, 8), (12, 16), (12, 16), (16, 16)]
    assert [layout(d, 2) for d in (384, 700, 768)] == [(6, 16), (12, 24), (12, 24)]
    pw, st = ctypes.c_int(0), ctypes.c_int(0)
    assert f(0, 0, ctypes.byref(pw), ctypes.byref(st)) == -3 and f(70000, 0, ctypes.byref(pw), ctypes.byref(st)) == -3
    assert f(768, 9, ctypes.byref(pw), ctypes.byref(st)) == -1 and f(768, 0, None, ctypes.byref(st)) == -2
    widths = _compiled_widths()
    for enc in (0, 1, 2):
        planes = 1 if enc == 1 else 2
        for d in list(range(1, 3300, 41)) + [64, 384, 768, 960, 1024, 1536, 3072, 65536]:
            nw = (d + 63) // 64
            pw, stride = layout(d, enc)
            assert nw <= pw <= nw + nw // 2 + 2 and 3 * pw <= 4 * nw or pw == nw
            nxt = next((w for w in widths if w >= nw), 0)               # the three encodings share the compiled widths
            assert pw == (nxt if nxt and 3 * nxt <= 4 * nw else nw)
            row = planes * pw
            assert stride >= row and (stride == row or stride % 2 == 0) and stride <= 4 * row + 16
            dense, chosen = mean_lines(row * 8, row * 8), mean_lines(row * 8, stride * 8)
            assert chosen <= dense
            if stride != row:
                assert chosen < dense                                      # padding only when it pays
                assert chosen == max(1, -(-row * 8 // 128))               # and then a row touches the fewest lines possible
            else:                                                          # no aligned stride would do better
                bytes_ = row * 8
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
    # the entry point with built-in scratch: same argument checks, and its own limit, all before any device call
    lib.qv_search_static.argtypes = [P, P, ctypes.c_int64, ctypes.c_int, ctypes.c_int, P, P, P, P]
    assert lib.qv_search_static(None, fake, 1, 1, 8, fake, fake, None, None) == -2
    assert lib.qv_search_static(h, fake, 1, 9, 8, fake, fake, None, None) == -4
    assert lib.qv_search_static(h, fake, 1, 1, 5000, fake, fake, None, None) == -5
    assert lib.qv_search_static(h, fake, 0, 1, 8, None, None, None, None) == 0
    assert lib.qv_search_static(h, fake, 10_000_000, 1, 8, fake, fake, None, None) == -10
    # split layout: only for the widths the kernel is compiled for; pointers checked
    w1, w2 = ctypes.c_int(0), ctypes.c_int(0)
    lib.qv_split_layout.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int)]
    assert lib.qv_split_layout(768, ctypes.byref(w1), ctypes.byref(w2)) == 0 and (w1.value, w2.value) == (16, 8)
    assert lib.qv_split_layout(1024, ctypes.byref(w1), ctypes.byref(w2)) == 0 and (w1.value, w2.value) == (16, 16)
    assert lib.qv_split_layout(1536, ctypes.byref(w1), ctypes.byref(w2)) == 0 and (w1.value, w2.value) == (32, 16)
    assert lib.qv_split_layout(384, ctypes.byref(w1), ctypes.byref(w2)) == -9
    assert lib.qv_split_layout(0, ctypes.byref(w1), ctypes.byref(w2)) == -3 and lib.qv_split_layout(768, None, None) == -2
    lib.qv_split_codes.argtypes = [P, ctypes.c_int64, ctypes.c_int, P, P, P]
    assert lib.qv_split_codes(fake, 5, 384, fake, fake, None) == -9 and lib.qv_split_codes(None, 5, 768, fake, fake, None) == -2
    assert lib.qv_split_codes(fake, -1, 768, fake, fake, None) == -1 and lib.qv_split_codes(None, 0, 768, None, None, None) == 0
    lib.qv_index_set_split_codes.argtypes = [P, P, P]
    assert lib.qv_index_set_split_codes(None, fake, fake) == -2
    assert lib.qv_index_set_split_codes(h, fake, fake) == -9          # the test index is 8-d
    assert lib.qv_index_set_split_codes(h, None, None) == 0
    lib.qv_index_set_tuning.argtypes = [P, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int]
    assert lib.qv_index_set_tuning(h, 512, 0, 0, 0, 0) == -1 and lib.qv_index_set_tuning(h, 0, 3, 0, 0, 0) == -1
    assert lib.qv_index_set_tuning(h, 0, 0, 16, 0, 0) == -1 and lib.qv_index_set_tuning(h, 8192, 4, 32, 0, 0) == 0
    assert lib.qv_index_set_tuning(h, 0, 0, 0, 3, 0) == -1 and lib.qv_index_set_tuning(h, 4096, 2, 0, 2, 0) == 0
    assert lib.qv_index_set_tuning(h, 0, 0, 0, 0, 4) == -1 and lib.qv_index_set_tuning(h, 0, 0, 0, 0, 3) == 0
    assert lib.qv_index_set_tuning(h, 0, 0, 0, 0, 1) == 0
    assert lib.qv_index_set_tuning(h, 0, 0, 0, 0, 2) == 0
    # where Stage 2 runs: inside the search kernel for beams of up to 128 over short code rows (d = 8 here), unless told otherwise
    lib.qv_index_rerank_fused.argtypes = [P, ctypes.c_int]
    assert lib.qv_index_rerank_fused(h, 64) == 1 and lib.qv_index_rerank_fused(h, 129) == 0
    assert lib.qv_index_set_tuning(h, 0, 0, 0, 0, 1) == 0 and lib.qv_index_rerank_fused(h, 64) == 0
    assert lib.qv_index_set_tuning(h, 0, 0, 0, 0, 0) == 0 and lib.qv_index_rerank_fused(h, 64) == 1
    assert lib.qv_index_rerank_fused(None, 64) == -2
    # layout of the index's codes (d = 8: one word per plane, two planes)
    lib.qv_index_set_code_layout.argtypes = [P, ctypes.c_int, ctypes.c_int]
    ok = lib.qv_index_set_code_layout
    assert ok(h, 0, 0) == 0 and ok(h, 1, 2) == 0 and ok(h, 1, 4) == 0 and ok(h, 2, 4) == 0 and ok(h, 3, 16) == 0
    assert ok(h, 1, 1) == -1 and ok(h, 1, 3) == -1 and ok(h, 2, 2) == -1 and ok(h, 4, 8) == -1 and ok(h, 0, 2) == -1
    assert ok(h, 1, 4096) == -1 and ok(None, 1, 2) == -2
    lib.qv_pad_codes.argtypes = [P, ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, P, P]
    assert lib.qv_pad_codes(fake, 5, 384, 0, 5, 16, fake, None) == -1      # planes shorter than the code's
    assert lib.qv_pad_codes(fake, 5, 384, 0, 6, 11, fake, None) == -1      # rows shorter than two planes
    assert lib.qv_pad_codes(fake, 5, 384, 0, 6, 13, fake, None) == -1      # odd
    assert lib.qv_pad_codes(fake, 5, 384, 0, 12, 24, fake, None) == -1     # planes more than half as wide again + 2
    assert lib.qv_pad_codes(fake, 5, 384, 7, 6, 16, fake, None) == -1      # unknown encoding
    assert lib.qv_pad_codes(fake, 5, 0, 0, 6, 16, fake, None) == -3
    assert lib.qv_pad_codes(None, 5, 384, 0, 6, 16, fake, None) == -2
    assert lib.qv_pad_codes(None, 0, 384, 0, 6, 16, None, None) == 0       # nothing to do
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
