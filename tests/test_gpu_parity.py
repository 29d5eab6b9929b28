"""GPU parity: the HIP library against the CPU oracle, element by element, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from tests import util
from workloads import datagen, graph

pytestmark = pytest.mark.gpu
E = util.E


@pytest.fixture(scope="module")
def qv():
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2605_02171_amd as m
    return m


def _special_vectors(d, rng):
    rows = []
    rows.append(np.full(d, 0.1, dtype=np.float32))                        # all equal: nothing is strong
    rows.append(np.zeros(d, dtype=np.float32))
    x = np.zeros(d, dtype=np.float32); x[::2] = -0.0; rows.append(x)
    base = np.float32(0.123456).view(np.uint32)
    ulps = rng.integers(-3, 4, size=d)
    x = (base + ulps).astype(np.uint32).view(np.float32) * rng.choice([-1.0, 1.0], size=d).astype(np.float32)
    rows.append(x.astype(np.float32))                                     # many values within ulps of the mean
    x = np.full(d, 0.3, dtype=np.float32); x[d // 2] = np.nextafter(np.float32(0.3), np.float32(1)); rows.append(x)
    expo = rng.integers(-140, 100, size=d)
    x = (rng.standard_normal(d) * np.exp2(expo.astype(np.float64))).astype(np.float32)
    rows.append(np.where(np.isfinite(x), x, 1.0).astype(np.float32))      # huge dynamic range
    x = rng.standard_normal(d).astype(np.float32) * np.float32(1e-41); rows.append(x)   # subnormals only
    x = np.full(d, 1e-45, dtype=np.float32); x[0] = 2e-45; rows.append(x)
    x = np.full(d, 3.0e38, dtype=np.float32); x[-1] = -3.4e38; rows.append(x)            # sum overflows float32
    return np.stack(rows)


@pytest.mark.parametrize("d", [1, 2, 63, 64, 65, 100, 128, 192, 200, 300, 384, 448, 512, 640, 768, 832, 960, 1000, 1200, 1280, 1472, 1536, 1600, 3072,
                               4096, 4100])
def test_encode_bit_exact(qv, d):
    rng = np.random.default_rng(100 + d)
    n = 523  # not a multiple of the vectors-per-workgroup
    x = rng.standard_normal((n, d)).astype(np.float32)
    x[:64] *= np.exp2(rng.integers(-30, 30, size=(64, 1))).astype(np.float32)
    x = np.concatenate([x, _special_vectors(d, rng)])
    want = oracle.encode(x, threads=8)
    got, status = qv.encode(torch.from_numpy(x).cuda(), want_status=True)
    assert (qv.to_numpy_u64(got) == want).all()
    assert (qv.to_numpy_u32(status) == 0).all()


def test_encode_workloads_bit_exact(qv):
    for name, n in (("C1", 10_000), ("C2", 20_000), ("C3", 20_000), ("C4", 5_000), ("C5", 20_000)):
        w = datagen.scaled(name, n=n, nq=10)
        x = datagen.make_base(w)
        want = oracle.encode(x, threads=8)
        got = qv.encode(torch.from_numpy(x).cuda())
        assert (qv.to_numpy_u64(got) == want).all(), name


def test_encode_flags_non_finite_and_empty_input(qv):
    x = np.ones((9, 70), dtype=np.float32)
    x[2, 5] = np.inf
    x[7, 69] = np.nan
    codes, status = qv.encode(torch.from_numpy(x).cuda(), want_status=True)
    st = qv.to_numpy_u32(status)
    assert st.tolist() == [0, 0, 1, 0, 0, 0, 0, 1, 0]
    ok = [0, 1, 3, 4, 5, 6, 8]
    assert (qv.to_numpy_u64(codes)[ok] == oracle.encode(x[ok])).all()
    empty = qv.encode(torch.empty((0, 70), dtype=torch.float32, device="cuda"))
    assert empty.shape == (0, 4)


@pytest.mark.parametrize("d", [40, 64, 100, 128, 250, 256, 384])
def test_encode_short_rows_share_a_wave(qv, d):
    """Widths at which one wave encodes several consecutive vectors: every count of leftover vectors, with
    vectors that need the exact redo (equal magnitudes) and non-finite ones anywhere among them."""
    rng = np.random.default_rng(d)
    for n in (1, 2, 3, 5, 7, 8, 9, 31, 33, 67):
        x = rng.standard_normal((n, d)).astype(np.float32)
        equal = rng.random(n) < 0.3
        x[equal] = np.float32(0.37) * rng.choice([-1.0, 1.0], size=(int(equal.sum()), d)).astype(np.float32)
        bad = (rng.random(n) < 0.2) & ~equal
        for i in np.flatnonzero(bad):
            x[i, rng.integers(0, d)] = [np.inf, -np.inf, np.nan][i % 3]
        codes, status = qv.encode(torch.from_numpy(x).cuda(), want_status=True)
        assert (qv.to_numpy_u32(status) == bad.astype(np.uint32)).all()
        if (~bad).any():
            want = oracle.encode(x[~bad], threads=2)
            assert (qv.to_numpy_u64(codes)[~bad] == want).all(), (d, n)
            assert (want[equal[~bad]][:, want.shape[1] // 2:] == 0).all()      # equal magnitudes: nothing is strong


@pytest.mark.parametrize("d", [1, 64, 100, 768, 3072])
def test_bq_distance_bit_exact(qv, d):
    rng = np.random.default_rng(7 + d)
    xa = rng.standard_normal((300, d)).astype(np.float32)
    xb = rng.standard_normal((200, d)).astype(np.float32)
    ca, cb = oracle.encode(xa), oracle.encode(xb)
    ia = rng.integers(0, 300, size=5000)
    ib = rng.integers(0, 200, size=5000)
    want = oracle.sm_distance_pairs(ca, ia, cb, ib, d)
    got = qv.bq_distance(qv.from_numpy_u64(ca), torch.from_numpy(ia).cuda(), qv.from_numpy_u64(cb),
                         torch.from_numpy(ib).cuda(), d)
    assert (qv.to_numpy_u32(got) == want).all()
    # identity and symmetry on the device as well
    same = qv.bq_distance(qv.from_numpy_u64(ca), torch.from_numpy(ia).cuda(), qv.from_numpy_u64(ca),
                          torch.from_numpy(ia).cuda(), d)
    assert (qv.to_numpy_u32(same) == 0).all()


def _run_both(qv, x, q, adj, entry, k, ef, visit_cap=256, visited_slots=0, lanes=0, table_format=0):
    """Oracle and GPU on the same inputs.  The GPU runs twice: with the visited set as a cache (the default;
    compared here, counters allowed to exceed the oracle's) and as a table that never forgets (returned)."""
    codes = oracle.encode(x, threads=8)
    ref = oracle.search(q, adj, codes, x, entry, k, ef, visit_cap=visit_cap, threads=8)
    xd = torch.from_numpy(x).cuda()
    gcodes = qv.encode(xd)
    assert (qv.to_numpy_u64(gcodes) == codes).all()
    index = qv.Index(qv.from_numpy_u32(adj), gcodes, xd, entry)
    qd = torch.from_numpy(q).cuda()
    if lanes or table_format:
        index.set_tuning(0, lanes, table_format)
    cached = qv.search(index, qd, k, ef, trace=True, visit_cap=visit_cap)
    torch.cuda.synchronize()
    _assert_search_equal(qv, ref, cached, exact_counters=False)
    plain = qv.search(index, qd, k, ef)          # no trace: the lists never leave the kernel when Stage 2 runs inside it
    torch.cuda.synchronize()
    assert torch.equal(plain.ids, cached.ids) and torch.equal(plain.scores, cached.scores)
    # Stage 2 as a kernel of its own and inside the search kernel (the default picks one of them by the row length)
    for rerank_mode in (qv.RERANK_SEPARATE, qv.RERANK_FUSED, qv.RERANK_TAIL):
        index.set_tuning(0, lanes, table_format, 0, rerank_mode)
        other = qv.search(index, qd, k, ef, trace=True, visit_cap=visit_cap)
        torch.cuda.synchronize()
        _assert_search_equal(qv, ref, other, exact_counters=False)
    index.set_tuning(visited_slots, lanes, table_format, qv.VISITED_EXACT)
    out = qv.search(index, qd, k, ef, trace=True, visit_cap=visit_cap)
    torch.cuda.synchronize()
    return ref, out


def _assert_search_equal(qv, ref, out, exact_counters=True):
    assert (qv.to_numpy_u32(out.cand_ids) == ref.cand_ids).all()
    assert (qv.to_numpy_u32(out.cand_dist) == ref.cand_dist).all()
    assert (qv.to_numpy_u32(out.n_cand) == ref.n_cand).all()
    assert (qv.to_numpy_u32(out.n_expanded) == ref.n_expanded).all()
    assert (qv.to_numpy_u32(out.visit_order) == ref.visit_order).all()
    ev = qv.to_numpy_u32(out.n_dist_evals)
    st = qv.to_numpy_u32(out.status)
    if exact_counters:
        assert (st == 0).all()
        assert (ev == ref.n_dist_evals).all()
    else:
        assert (ev >= ref.n_dist_evals).all()
        assert (ev[(st & 2) == 0] == ref.n_dist_evals[(st & 2) == 0]).all()
    util.assert_topk_matches(qv.to_numpy_u32(out.ids), out.scores.cpu().numpy(), ref.ids, ref.scores)


def test_search_tiny_workload_all_queries(qv):
    w = datagen.WORKLOADS["C1"]
    x, q = datagen.make_base(w), datagen.make_queries(w)
    adj, entry = graph.build_graph(x, w.R, w.L, w.alpha)
    ref, out = _run_both(qv, x, q, adj, entry, w.k, 64)
    _assert_search_equal(qv, ref, out)


@pytest.mark.parametrize("d,R,ef,k", [
    (100, 10, 1, 1), (100, 10, 5, 5), (128, 32, 64, 10), (200, 70, 65, 10), (64, 64, 128, 128),
    (384, 64, 16, 10), (768, 64, 32, 10), (512, 17, 200, 50), (1024, 64, 64, 10), (130, 130, 300, 7),
])
def test_search_random_graphs_bit_exact(qv, d, R, ef, k):
    rng = np.random.default_rng(d * 1000 + R)
    n, nq = 3000, 37
    x = rng.standard_normal((n, d)).astype(np.float32)
    q = rng.standard_normal((nq, d)).astype(np.float32)
    adj = datagen.random_regular_graph(n, R, seed=d + R, fill=0.85)
    ref, out = _run_both(qv, x, q, adj, entry=5, k=k, ef=ef, visit_cap=400)
    _assert_search_equal(qv, ref, out, exact_counters=False)


@pytest.mark.parametrize("lanes", [1, 2, 4, 8, 16])
def test_search_every_gather_width(qv, lanes):
    w = datagen.scaled("C2", n=6000, nq=25)
    x, q = datagen.make_base(w), datagen.make_queries(w)
    adj, entry = graph.build_graph(x, 64, 64, 1.2)
    ref, out = _run_both(qv, x, q, adj, entry, 10, 48, lanes=lanes)
    _assert_search_equal(qv, ref, out)


@pytest.mark.parametrize("table_format", [0, 32])
def test_search_full_visited_table_keeps_results_exact(qv, table_format):
    # a deliberately small visited table: it fills up, nodes get re-evaluated, the lists must not change
    w = datagen.scaled("C2", n=20_000, nq=40)
    x, q = datagen.make_base(w), datagen.make_queries(w)
    adj, entry = graph.build_graph(x, 64, 64, 1.2)
    ref, out = _run_both(qv, x, q, adj, entry, 10, 128, visit_cap=300, visited_slots=1024, table_format=table_format)
    st = qv.to_numpy_u32(out.status)
    assert (st & 2).any(), "the test is meant to overflow the table"
    _assert_search_equal(qv, ref, out, exact_counters=False)


@pytest.mark.parametrize("table_format", [0, 32])
def test_search_both_visited_table_formats(qv, table_format):
    w = datagen.scaled("C3", n=30_000, nq=60)
    x, q = datagen.make_base(w), datagen.make_queries(w)
    adj, entry = graph.build_graph(x, 64, 48, 1.2)
    ref, out = _run_both(qv, x, q, adj, entry, 10, 64, visit_cap=300, table_format=table_format)
    _assert_search_equal(qv, ref, out)


def test_search_visited_table_in_several_parts(qv):
    # n > 65535: the 16-bit table is cut into parts (three here, of a size that is not a power of two)
    w = datagen.scaled("C3", n=150_000, nq=80)
    x, q = datagen.make_base(w), datagen.make_queries(w)
    adj, entry = graph.build_graph(x, 64, 32, 1.2)
    ref, out = _run_both(qv, x, q, adj, entry, 10, 64, visit_cap=300)
    _assert_search_equal(qv, ref, out)


def test_search_small_table_in_eight_parts_overflows_gracefully(qv):
    # 1024 slots in 8 parts of 128: single parts fill up before the table does
    rng = np.random.default_rng(77)
    n, d = 500_000, 64
    x = rng.standard_normal((n, d)).astype(np.float32)
    q = rng.standard_normal((64, d)).astype(np.float32)
    adj = datagen.random_regular_graph(n, 16, seed=9)
    ref, out = _run_both(qv, x, q, adj, entry=11, k=10, ef=128, visit_cap=300, visited_slots=1024)
    assert (qv.to_numpy_u32(out.status) & 2).all()
    _assert_search_equal(qv, ref, out, exact_counters=False)


@pytest.mark.parametrize("table_format,slots,ef", [(0, 1024, 64), (32, 1024, 64), (0, 1024, 300), (32, 2048, 128),
                                                    (0, 3072, 1024)])
def test_search_tiny_visited_cache_keeps_results_exact(qv, table_format, slots, ef):
    # a cache far smaller than the set of evaluated nodes: ids displace each other all the time, nodes come
    # back and are evaluated again; lists, distances and the expansion order must not change
    w = datagen.scaled("C2", n=30_000, nq=48)
    x, q = datagen.make_base(w), datagen.make_queries(w)
    adj, entry = graph.build_graph(x, 64, 64, 1.2)
    adj[::7, 5] = adj[::7, 9]                   # duplicate edges and self loops on top
    adj[::11, 3] = np.arange(0, w.n, 11, dtype=np.uint32)
    codes = oracle.encode(x, threads=8)
    ref = oracle.search(q, adj, codes, x, entry, 10, ef, visit_cap=1200, threads=8)
    xd = torch.from_numpy(x).cuda()
    index = qv.Index(qv.from_numpy_u32(adj), qv.encode(xd), xd, entry)
    index.set_tuning(slots, 0, table_format, qv.VISITED_CACHE)
    out = qv.search(index, torch.from_numpy(q).cuda(), 10, ef, trace=True, visit_cap=1200)
    torch.cuda.synchronize()
    assert (qv.to_numpy_u32(out.status) & 2).all(), "the test is meant to displace ids"
    assert (qv.to_numpy_u32(out.n_dist_evals) > ref.n_dist_evals).any()
    _assert_search_equal(qv, ref, out, exact_counters=False)


@pytest.mark.parametrize("table_format", [0, 32])
def test_search_rows_that_name_nodes_several_times(qv, table_format):
    # adjacency rows drawn with replacement from a few nodes: most rows name a node two, three or more times, in
    # places that fall into the same expansion; the second occurrence must not be evaluated (counts equal the
    # oracle's wherever the cache forgot nothing) and must never reach the list twice
    rng = np.random.default_rng(404)
    n, d, R = 4000, 256, 64
    x = rng.standard_normal((n, d)).astype(np.float32)
    q = rng.standard_normal((50, d)).astype(np.float32)
    near = rng.integers(0, n, size=(n, 40))
    adj = np.take_along_axis(near, rng.integers(0, 40, size=(n, R)), axis=1).astype(np.uint32)
    assert max(len(set(r.tolist())) for r in adj[:200]) < R - 15
    codes = oracle.encode(x, threads=8)
    xd = torch.from_numpy(x).cuda()
    index = qv.Index(qv.from_numpy_u32(adj), qv.encode(xd), xd, 9)
    for ef in (4, 64, 200):
        ref = oracle.search(q, adj, codes, x, 9, min(10, ef), ef, visit_cap=600, threads=8)
        for mode in (qv.VISITED_CACHE, qv.VISITED_EXACT):
            index.set_tuning(0, 0, table_format, mode)
            out = qv.search(index, torch.from_numpy(q).cuda(), min(10, ef), ef, trace=True, visit_cap=600)
            torch.cuda.synchronize()
            _assert_search_equal(qv, ref, out, exact_counters=False)
            if ef == 4:   # few enough insertions that the cache forgets nothing for many queries (a repeated node uses
                # up places in its bucket, so the flag comes early on such rows): their counts were compared above
                assert ((qv.to_numpy_u32(out.status) & 2) == 0).mean() > 0.2


def test_search_visited_cache_on_a_graph_with_many_parts(qv):
    # 500,000 nodes: the 16-bit cache is cut into eight parts of 64 buckets at the default 4096 slots
    rng = np.random.default_rng(78)
    n, d = 500_000, 64
    x = rng.standard_normal((n, d)).astype(np.float32)
    q = rng.standard_normal((64, d)).astype(np.float32)
    adj = datagen.random_regular_graph(n, 16, seed=10)
    codes = oracle.encode(x, threads=8)
    ref = oracle.search(q, adj, codes, x, 11, 10, 128, visit_cap=300, threads=8)
    xd = torch.from_numpy(x).cuda()
    index = qv.Index(qv.from_numpy_u32(adj), qv.encode(xd), xd, 11)
    for slots in (0, 1024):
        index.set_tuning(slots, 0, 0, qv.VISITED_CACHE)
        out = qv.search(index, torch.from_numpy(q).cuda(), 10, 128, trace=True, visit_cap=300)
        torch.cuda.synchronize()
        _assert_search_equal(qv, ref, out, exact_counters=False)


@pytest.mark.parametrize("ef", [256, 512, 1024])
def test_search_wide_beams(qv, ef):
    # beams beyond two registers per lane; at ef = 1024 the visited table is capped by the 64 KB of LDS
    w = datagen.scaled("C2", n=40_000, nq=24)
    x, q = datagen.make_base(w), datagen.make_queries(w)
    adj, entry = graph.build_graph(x, 64, 48, 1.2)
    ref, out = _run_both(qv, x, q, adj, entry, 10, ef, visit_cap=1200)
    _assert_search_equal(qv, ref, out, exact_counters=False)


@pytest.mark.parametrize("nq", [4095, 4096, 4097, 4608, 5000])
def test_search_batches_around_the_launch_order_threshold(qv, nq):
    # from 4,096 queries on, workgroups pick their queries through a launch order (ranked per 512-query slice and
    # interleaved; the last slice may be ragged): every query must still be searched exactly once
    rng = np.random.default_rng(nq)
    n, d = 4000, 64
    x = rng.standard_normal((n, d)).astype(np.float32)
    q = rng.standard_normal((nq, d)).astype(np.float32)
    q[::97] = q[0]                               # equal queries: equal distances to the entry node
    adj = datagen.random_regular_graph(n, 12, seed=3)
    ref, out = _run_both(qv, x, q, adj, entry=17, k=5, ef=24, visit_cap=64)
    _assert_search_equal(qv, ref, out, exact_counters=False)


@pytest.mark.parametrize("d,layout,enc,nq", [(384, None, 0, 37), (960, None, 0, 37), (300, None, 0, 37), (448, None, 0, 37),
                                             (1100, None, 0, 37), (2048, (32, 80), 0, 37), (200, (6, 12), 0, 37),
                                             (100, (2, 6), 0, 37), (100, (4, 8), 0, 37), (768, (12, 32), 0, 37),
                                             (768, (16, 32), 0, 37), (960, (15, 32), 0, 37), (1000, (24, 48), 0, 37),
                                             (192, None, 1, 37), (700, None, 1, 37), (384, None, 2, 37), (700, None, 2, 37),
                                             (384, None, 0, 4200), (960, None, 0, 4200)])
def test_search_with_another_code_layout(qv, d, layout, enc, nq):
    """Index codes with planes padded by zero words and rows further apart than their length: the re-laid-out
    copy holds the dense code's words where the layout says, zeros elsewhere, and the search through it returns
    what the oracle returns on dense rows."""
    rng = np.random.default_rng(d + 7 * enc)
    n, R, ef, k = 3000, 32, 48, 10
    x = rng.standard_normal((n, d)).astype(np.float32)
    q = rng.standard_normal((nq, d)).astype(np.float32)
    adj = datagen.random_regular_graph(n, R, seed=d, fill=0.9)
    codes = oracle.encode(x, threads=8, enc=enc)
    ref = oracle.search(q, adj, codes, x, 11, k, ef, visit_cap=200, threads=8, enc=enc)
    xd = torch.from_numpy(x).cuda()
    nw, planes = (d + 63) // 64, (1 if enc == qv.ENC_SIGN1 else 2)
    if layout is None:
        layout = qv.code_layout(d, enc)
        assert layout != (nw, planes * nw)          # these widths are the ones another layout helps
    pw, stride = layout
    padded = qv.pad_codes(qv.encode(xd, enc=enc), d, layout, enc=enc)
    got = qv.to_numpy_u64(padded)
    assert got.shape == (n, stride)
    want = np.zeros((n, stride), dtype=np.uint64)
    for p in range(planes):
        want[:, p * pw:p * pw + nw] = codes[:, p * nw:(p + 1) * nw]
    assert (got == want).all()
    index = qv.Index(qv.from_numpy_u32(adj), padded, xd, 11, enc=enc, layout=layout)
    qd = torch.from_numpy(q).cuda()
    for mode in (qv.VISITED_CACHE, qv.VISITED_EXACT):
        index.set_tuning(0, 0, 0, mode)
        out = qv.search(index, qd, k, ef, trace=True, visit_cap=200)
        torch.cuda.synchronize()
        _assert_search_equal(qv, ref, out, exact_counters=False)


def test_search_degenerate_graphs(qv):
    rng = np.random.default_rng(3)
    n, d = 500, 96
    x = rng.standard_normal((n, d)).astype(np.float32)
    q = rng.standard_normal((9, d)).astype(np.float32)
    # no edges at all: the list is the entry node
    adj = np.full((n, 8), E, dtype=np.uint32)
    ref, out = _run_both(qv, x, q, adj, entry=7, k=3, ef=8)
    _assert_search_equal(qv, ref, out)
    assert (qv.to_numpy_u32(out.ids)[:, 0] == 7).all() and (qv.to_numpy_u32(out.ids)[:, 1:] == E).all()
    # self loops, duplicate edges, a chain
    adj = np.full((n, 8), E, dtype=np.uint32)
    adj[:, 0] = np.arange(n)
    adj[:, 1] = (np.arange(n) + 1) % n
    adj[:, 2] = adj[:, 1]
    adj[:, 5] = (np.arange(n) * 7 + 3) % n
    ref, out = _run_both(qv, x, q, adj, entry=0, k=4, ef=10, visit_cap=600)
    _assert_search_equal(qv, ref, out)
    # a single node
    ref, out = _run_both(qv, x[:1], q, np.full((1, 4), E, dtype=np.uint32), entry=0, k=1, ef=4)
    _assert_search_equal(qv, ref, out)


def test_search_skips_edges_to_missing_nodes_and_reports_them(qv):
    rng = np.random.default_rng(4)
    n, d = 300, 64
    x = rng.standard_normal((n, d)).astype(np.float32)
    q = rng.standard_normal((5, d)).astype(np.float32)
    adj = datagen.random_regular_graph(n, 6, seed=1)
    bad = adj.copy()
    bad[:, 3] = np.uint32(n + 5)                       # every row has one edge to a node that does not exist
    clean = adj.copy()
    clean[:, 3] = E
    codes = oracle.encode(x)
    ref = oracle.search(q, clean, codes, x, 0, 5, 20, visit_cap=300)
    xd = torch.from_numpy(x).cuda()
    index = qv.Index(qv.from_numpy_u32(bad), qv.encode(xd), xd, 0)
    out = qv.search(index, torch.from_numpy(q).cuda(), 5, 20, trace=True, visit_cap=300)
    assert (qv.to_numpy_u32(out.cand_ids) == ref.cand_ids).all()
    assert (qv.to_numpy_u32(out.status) & 4).all()


def test_empty_batch_and_argument_errors(qv):
    rng = np.random.default_rng(5)
    x = rng.standard_normal((50, 64)).astype(np.float32)
    xd = torch.from_numpy(x).cuda()
    index = qv.Index(qv.from_numpy_u32(datagen.random_regular_graph(50, 4, 1)), qv.encode(xd), xd, 0)
    out = qv.search(index, torch.empty((0, 64), dtype=torch.float32, device="cuda"), 3, 8)
    assert out.ids.shape == (0, 3)
    qd = xd[:4].contiguous()
    with pytest.raises(qv.QuiverError) as e:
        qv.search(index, qd, 9, 8)
    assert e.value.code == -4
    with pytest.raises(qv.QuiverError) as e:
        qv.search(index, qd, 1, qv.MAX_EF + 1)
    assert e.value.code == -5
    with pytest.raises(qv.QuiverError) as e:
        qv.search(index, qd, 1, 8, workspace=torch.empty(16, dtype=torch.uint8, device="cuda"))
    assert e.value.code == -6
    with pytest.raises(qv.QuiverError):
        qv.Index(qv.from_numpy_u32(datagen.random_regular_graph(50, 4, 1)), qv.encode(xd), xd, 50)


@pytest.mark.parametrize("name,n,ef", [("C2", 50_000, 64), ("C2", 50_000, 128), ("C3", 50_000, 64),
                                       ("C4", 12_000, 64), ("C5", 50_000, 64)])
def test_search_workload_shapes_reduced_n(qv, name, n, ef):
    w = datagen.scaled(name, n=n, nq=200)
    x, q = datagen.make_base(w), datagen.make_queries(w)
    adj, entry = graph.build_graph(x, w.R, 64, w.alpha)
    ref, out = _run_both(qv, x, q, adj, entry, w.k, ef, visit_cap=400)
    _assert_search_equal(qv, ref, out)


def test_search_with_cold_vectors_in_pinned_host_memory(qv):
    # the float32 vectors are only read by the rerank; they may stay in host memory the device can address
    w = datagen.scaled("C2", n=30_000, nq=64)
    x, q = datagen.make_base(w), datagen.make_queries(w)
    adj, entry = graph.build_graph(x, 64, 48, 1.2)
    codes = oracle.encode(x, threads=8)
    ref = oracle.search(q, adj, codes, x, entry, 10, 64, visit_cap=256, threads=8)
    cold = torch.empty(x.shape, dtype=torch.float32, pin_memory=True)
    cold.copy_(torch.from_numpy(x))
    index = qv.Index(qv.from_numpy_u32(adj), qv.from_numpy_u64(codes), cold, entry)
    out = qv.search(index, torch.from_numpy(q).cuda(), 10, 64, trace=True, visit_cap=256)
    torch.cuda.synchronize()
    _assert_search_equal(qv, ref, out, exact_counters=False)


@pytest.mark.parametrize("rerank_mode", [0, 3])
def test_search_replays_from_a_captured_graph(qv, rerank_mode):
    # qv_search allocates nothing and records only kernels: with caller-owned workspace and outputs the whole call
    # can be captured once and replayed on new query contents; every replay must equal an eager call
    w = datagen.scaled("C3", n=20_000, nq=4500)          # above the launch-order threshold
    x = datagen.make_base(w)
    adj, entry = graph.build_graph(x, 32, 32, 1.2)
    xd = torch.from_numpy(x).cuda()
    index = qv.Index(qv.from_numpy_u32(adj), qv.encode(xd), xd, entry)
    index.set_tuning(0, 0, 0, 0, rerank_mode)   # 3: Stage 2 by other waves of the search launch (tickets and flags in the workspace)
    k, ef = 10, 48
    rng = np.random.default_rng(5)
    static_q = torch.zeros((w.nq, w.d), dtype=torch.float32, device="cuda")
    ws = torch.empty((qv.search_workspace_bytes(w.nq, w.d, k, ef),), dtype=torch.uint8, device="cuda")
    i32 = lambda *s: torch.zeros(s, dtype=torch.int32, device="cuda")
    out = qv.SearchOutput(i32(w.nq, k), torch.zeros((w.nq, k), dtype=torch.float32, device="cuda"),
                          cand_ids=i32(w.nq, ef), cand_dist=i32(w.nq, ef), n_cand=i32(w.nq), n_expanded=i32(w.nq),
                          n_dist_evals=i32(w.nq), status=i32(w.nq))
    qv.search(index, static_q, k, ef, workspace=ws, out=out)             # warm-up outside the capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        qv.search(index, static_q, k, ef, workspace=ws, out=out)
    for rep in range(3):
        q = torch.from_numpy(rng.standard_normal((w.nq, w.d)).astype(np.float32)).cuda()
        eager = qv.search(index, q, k, ef, trace=True)                   # the program's own eager work between replays
        torch.cuda.synchronize()
        static_q.copy_(q)
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.cand_ids, eager.cand_ids) and torch.equal(out.cand_dist, eager.cand_dist), rep
        assert torch.equal(out.ids, eager.ids) and torch.equal(out.scores, eager.scores), rep
        assert torch.equal(out.n_expanded, eager.n_expanded), rep


@pytest.mark.parametrize("rerank_mode", [0, 3])
def test_searches_on_two_streams_at_once(qv, rerank_mode):
    # the index is read-only and all scratch lives in the caller's workspace: two searches with separate workspaces
    # may run on different streams at the same time (default stream priority); each must equal its own solo run
    w = datagen.scaled("C3", n=20_000, nq=4500)
    x = datagen.make_base(w)
    adj, entry = graph.build_graph(x, 32, 32, 1.2)
    xd = torch.from_numpy(x).cuda()
    index = qv.Index(qv.from_numpy_u32(adj), qv.encode(xd), xd, entry)
    index.set_tuning(0, 0, 0, 0, rerank_mode)
    rng = np.random.default_rng(11)
    qa = torch.from_numpy(rng.standard_normal((w.nq, w.d)).astype(np.float32)).cuda()
    qb = torch.from_numpy(rng.standard_normal((1500, w.d)).astype(np.float32)).cuda()
    solo_a = qv.search(index, qa, 10, 48, trace=True)
    solo_b = qv.search(index, qb, 5, 100, trace=True)
    torch.cuda.synchronize()
    ref = oracle.search(qb.cpu().numpy()[:50], adj, oracle.encode(x, threads=8), x, entry, 5, 100, threads=8)
    assert (qv.to_numpy_u32(solo_b.cand_ids)[:50] == ref.cand_ids).all()
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    for rep in range(3):
        with torch.cuda.stream(sa):
            out_a = qv.search(index, qa, 10, 48, trace=True)
        with torch.cuda.stream(sb):
            out_b = qv.search(index, qb, 5, 100, trace=True)
        sa.synchronize(); sb.synchronize()
        for got, want in ((out_a, solo_a), (out_b, solo_b)):
            assert torch.equal(got.cand_ids, want.cand_ids) and torch.equal(got.cand_dist, want.cand_dist), rep
            assert torch.equal(got.ids, want.ids) and torch.equal(got.scores, want.scores), rep
            assert torch.equal(got.n_expanded, want.n_expanded), rep


@pytest.mark.parametrize("d,ef", [(128, 64), (768, 32), (100, 200)])
def test_search_reports_non_finite_queries_and_leaves_the_rest_exact(qv, d, ef):
    # queries with NaN, +Inf and -Inf mixed into a batch: each of them comes back empty and flagged, in both forms of
    # Stage 2; every other query equals the oracle's result on the finite queries alone (the oracle rejects the others)
    rng = np.random.default_rng(d + ef)
    n, nq, k = 4000, 41, 10
    x = rng.standard_normal((n, d)).astype(np.float32)
    q = rng.standard_normal((nq, d)).astype(np.float32)
    adj = datagen.random_regular_graph(n, 32, seed=d, fill=0.9)
    bad = {0: np.nan, 7: np.inf, 8: -np.inf, 23: np.nan, nq - 1: np.inf}
    for i, v in bad.items():
        q[i, (i * 13) % d] = v
    q[23, :] = np.nan
    good = np.array([i for i in range(nq) if i not in bad])
    codes = oracle.encode(x, threads=8)
    with pytest.raises(oracle.OracleError):
        oracle.search(q[:1], adj, codes, x, 5, k, ef)
    ref = oracle.search(q[good], adj, codes, x, 5, k, ef, visit_cap=300, threads=8)
    xd = torch.from_numpy(x).cuda()
    index = qv.Index(qv.from_numpy_u32(adj), qv.encode(xd), xd, 5)
    qd = torch.from_numpy(q).cuda()
    for rerank_mode in (qv.RERANK_SEPARATE, qv.RERANK_FUSED, qv.RERANK_TAIL, 0):
        for visited_mode in (qv.VISITED_EXACT, qv.VISITED_CACHE):
            index.set_tuning(0, 0, 0, visited_mode, rerank_mode)
            for trace in (True, False):
                out = qv.search(index, qd, k, ef, trace=trace, visit_cap=300)
                torch.cuda.synchronize()
                ids, scores = qv.to_numpy_u32(out.ids), out.scores.cpu().numpy()
                for i in bad:
                    assert (ids[i] == E).all() and np.isneginf(scores[i]).all(), (i, rerank_mode)
                util.assert_topk_matches(ids[good], scores[good], ref.ids, ref.scores)
                if not trace:
                    continue
                st = qv.to_numpy_u32(out.status)
                assert (st[list(bad)] == qv.STATUS_NONFINITE).all() and (st[good] & qv.STATUS_NONFINITE == 0).all()
                for name in ("cand_ids", "cand_dist", "visit_order"):
                    got = qv.to_numpy_u32(getattr(out, name))
                    assert (got[list(bad)] == E).all(), name
                    assert (got[good] == getattr(ref, name)).all(), name
                for name in ("n_cand", "n_expanded", "n_dist_evals"):
                    assert (qv.to_numpy_u32(getattr(out, name))[list(bad)] == 0).all(), name
                assert (qv.to_numpy_u32(out.n_cand)[good] == ref.n_cand).all()
                assert (qv.to_numpy_u32(out.n_expanded)[good] == ref.n_expanded).all()


def test_rerank_puts_non_finite_stored_vectors_last(qv):
    # an index whose float32 rows hold Inf / NaN (their codes come from clean data): those list members score -inf
    # and follow every finite score, ordered by id, in both forms of Stage 2
    rng = np.random.default_rng(5)
    n, d, nq, ef = 300, 128, 9, 300
    x = rng.standard_normal((n, d)).astype(np.float32)
    q = rng.standard_normal((nq, d)).astype(np.float32)
    adj = np.stack([(np.arange(n) + s) % n for s in (1, 2, 5, 11, 31, 67)], axis=1).astype(np.uint32)
    codes = qv.from_numpy_u64(oracle.encode(x))
    dirty = x.copy()
    dirty[17, 3], dirty[200, 0], dirty[5, 127] = np.nan, np.inf, -np.inf
    xd = torch.from_numpy(dirty).cuda()
    index = qv.Index(qv.from_numpy_u32(adj), codes, xd, 0)
    ref = oracle.search(q, adj, oracle.encode(x), x, 0, n, ef)
    for ef_run, mode in ((ef, qv.RERANK_SEPARATE), (128, qv.RERANK_FUSED), (128, qv.RERANK_TAIL), (128, qv.RERANK_SEPARATE)):
        index.set_tuning(0, 0, 0, qv.VISITED_EXACT, mode)
        k = ef_run if ef_run < n else n
        out = qv.search(index, torch.from_numpy(q).cuda(), k, ef_run, trace=True)
        torch.cuda.synchronize()
        ids, scores, cand = qv.to_numpy_u32(out.ids), out.scores.cpu().numpy(), qv.to_numpy_u32(out.cand_ids)
        for i in range(nq):
            members = set(cand[i][cand[i] != E].tolist())
            tail = sorted(members & {5, 17, 200})
            got_tail = ids[i][np.isneginf(scores[i]) & (ids[i] != E)].tolist()
            assert got_tail == tail, (i, mode)
            if tail:
                first = int(np.flatnonzero(np.isneginf(scores[i]))[0])
                assert np.isfinite(scores[i][:first]).all() and (np.diff(scores[i][:first]) <= 0).all()
        if ef_run == ef:     # the whole graph is in the list: the finite part is the oracle's ranking without the three rows
            keep = ~np.isin(ref.ids, [5, 17, 200])
            want_ids = np.stack([r[m] for r, m in zip(ref.ids, keep)])
            want_scores = np.stack([r[m] for r, m in zip(ref.scores, keep)])
            util.assert_topk_matches(ids[:, :n - 3], scores[:, :n - 3], want_ids, want_scores)


@pytest.mark.parametrize("ef,k", [(64, 1), (64, 4), (129, 8), (300, 10), (300, 18), (300, 19), (1024, 64), (1024, 65)])
def test_rerank_kernel_takes_few_of_many_with_ties(qv, ef, k):
    # Stage 2 as a kernel of its own picks a small k out of a long list in k rounds, a larger one by ranking all:
    # both sides of that switch (k * 16 <= list length), on vectors that repeat (equal scores: the smaller id comes
    # first), that point away from the query (negative scores), and with rows that hold NaN / Inf (they come last)
    rng = np.random.default_rng(ef * 100 + k)
    n, d, nq = 1100, 192, 21
    base = rng.standard_normal((40, d)).astype(np.float32)
    x = base[rng.integers(0, 40, size=n)] * rng.choice([1.0, -1.0, 2.0], size=(n, 1)).astype(np.float32)
    q = (base[rng.integers(0, 40, size=nq)] + 0.05 * rng.standard_normal((nq, d))).astype(np.float32)
    adj = np.stack([(np.arange(n) * 7 + s) % n for s in range(1, 33)], axis=1).astype(np.uint32)
    codes = oracle.encode(x)
    ref = oracle.search(q, adj, codes, x, 3, k, ef)
    xd = torch.from_numpy(x).cuda()
    index = qv.Index(qv.from_numpy_u32(adj), qv.from_numpy_u64(codes), xd, 3)
    index.set_tuning(0, 0, 0, 0, qv.RERANK_SEPARATE)
    out = qv.search(index, torch.from_numpy(q).cuda(), k, ef, trace=True)
    torch.cuda.synchronize()
    assert (qv.to_numpy_u32(out.cand_ids) == ref.cand_ids).all()
    ids, scores = qv.to_numpy_u32(out.ids), out.scores.cpu().numpy()
    util.assert_topk_matches(ids, scores, ref.ids, ref.scores)
    # exact ties are decided by id: among the results of one query, equal scores come with ascending ids, and a
    # list member left out at the k-th score has a larger id than the ones taken at that score
    exact = x.astype(np.float64)
    for i in range(nq):
        assert (np.diff(scores[i]) <= 0).all()
        for r in range(k - 1):
            if scores[i][r] == scores[i][r + 1]:
                assert ids[i][r] < ids[i][r + 1], (i, r)
        members = ref.cand_ids[i][ref.cand_ids[i] != E]
        left_out = np.setdiff1d(members, ids[i])
        qq = q[i].astype(np.float64)
        cos = exact[left_out] @ qq / (np.linalg.norm(exact[left_out], axis=1) * np.linalg.norm(qq))
        assert (cos <= float(scores[i][-1]) * (1 + 2e-5 * np.sign(scores[i][-1])) + 1e-6).all()
    # the same lists with three rows spoiled: they score -inf and come last, by id
    dirty = x.copy()
    spoiled = sorted(int(v) for v in ref.cand_ids[0][:3])
    dirty[spoiled[0], 1], dirty[spoiled[1], 0], dirty[spoiled[2], d - 1] = np.nan, np.inf, -np.inf
    index2 = qv.Index(qv.from_numpy_u32(adj), qv.from_numpy_u64(codes), torch.from_numpy(dirty).cuda(), 3)
    index2.set_tuning(0, 0, 0, 0, qv.RERANK_SEPARATE)
    k_all = min(ef, int(ref.n_cand[0]))
    out2 = qv.search(index2, torch.from_numpy(q[:1]).cuda(), k_all, ef, trace=True)
    torch.cuda.synchronize()
    ids2, sc2 = qv.to_numpy_u32(out2.ids)[0], out2.scores.cpu().numpy()[0]
    assert ids2[-3:].tolist() == spoiled and np.isneginf(sc2[-3:]).all() and np.isfinite(sc2[:-3]).all()
    few = qv.search(index2, torch.from_numpy(q[:1]).cuda(), k, ef)
    torch.cuda.synchronize()
    keep = min(k, k_all - 3)
    assert (qv.to_numpy_u32(few.ids)[0][:keep] == ids2[:keep]).all() and (few.scores.cpu().numpy()[0][:keep] == sc2[:keep]).all()


@pytest.mark.parametrize("d,R,ef,k,n", [(768, 64, 64, 10, 20_000), (768, 64, 16, 10, 3_000), (768, 32, 200, 50, 20_000),
                                        (1024, 64, 64, 10, 8_000), (1536, 48, 100, 10, 5_000), (768, 70, 1024, 100, 9_000),
                                        (768, 64, 1, 1, 6_000)])
def test_search_split_code_layout_is_bit_exact(qv, d, R, ef, k, n):
    # the index's code rows in the split layout (sign plane first; the rest of the magnitude plane only for neighbours
    # the sign-plane bound lets through): lists, distances, expansion order and counters as with dense rows
    w = datagen.scaled("H2", n=n, nq=45, d=d)
    x, q = datagen.make_base(w), datagen.make_queries(w)
    rng = np.random.default_rng(d + ef)
    x[n // 2: n // 2 + 30] = x[:30]               # repeated vectors: distance ties at the list's edge
    adj = datagen.random_regular_graph(n, R, seed=d + R, fill=0.9) if R != 64 else graph.build_graph(x, 64, 64, 1.2)[0]
    entry = 7
    codes = oracle.encode(x, threads=8)
    ref = oracle.search(q, adj, codes, x, entry, k, ef, visit_cap=1300, threads=8)
    xd = torch.from_numpy(x).cuda()
    gcodes = qv.encode(xd)
    lay = qv.split_layout(d)
    nw = (d + 63) // 64
    assert lay is not None and sum(lay) == 2 * nw and lay[0] % 16 == 0
    s1, s2 = qv.split_codes(gcodes, d)
    # the two arrays hold the same words: sign plane, then magnitude words in order
    h1, h2 = qv.to_numpy_u64(s1), qv.to_numpy_u64(s2)
    k1 = lay[0] - nw
    assert (h1[:, :nw] == codes[:, :nw]).all() and (h1[:, nw:] == codes[:, nw:nw + k1]).all()
    assert (h2 == codes[:, nw + k1:]).all()
    index = qv.Index(qv.from_numpy_u32(adj), gcodes, xd, entry)
    index.set_split_codes((s1, s2))
    qd = torch.from_numpy(q).cuda()
    for visited_mode in (qv.VISITED_EXACT, qv.VISITED_CACHE):
        for rerank_mode in (qv.RERANK_SEPARATE, qv.RERANK_FUSED, qv.RERANK_TAIL):
            index.set_tuning(1024 if visited_mode == qv.VISITED_CACHE and ef <= 64 else 0, 0, 0, visited_mode, rerank_mode)
            out = qv.search(index, qd, k, ef, trace=True, visit_cap=1300)
            torch.cuda.synchronize()
            _assert_search_equal(qv, ref, out, exact_counters=False)
    index.set_tuning(0, 0, 32, 0, 0)              # 32-bit visited entries, everything else by default
    out = qv.search(index, qd, k, ef, trace=True, visit_cap=1300)
    torch.cuda.synchronize()
    _assert_search_equal(qv, ref, out, exact_counters=False)
    index.set_split_codes(None)
    index.set_tuning(0, 0, 0, qv.VISITED_EXACT)
    out = qv.search(index, qd, k, ef, trace=True, visit_cap=1300)
    torch.cuda.synchronize()
    _assert_search_equal(qv, ref, out, exact_counters=False)


def test_split_layout_applies_to_long_rows_only(qv):
    for d in (64, 384, 512, 2048, 3072):
        assert qv.split_layout(d) is None
    assert qv.split_layout(768) == (16, 8) and qv.split_layout(1024) == (16, 16) and qv.split_layout(1536) == (32, 16)
    codes = torch.zeros((10, 12), dtype=torch.int64, device="cuda")
    with pytest.raises(qv.QuiverError) as e:
        qv.split_codes(codes, 384)
    assert e.value.code == -9
