"""Pins for the oracle's beam search and rerank (paper Sec. 3.3, Stage 1 and Stage 2)."""
import numpy as np
import pytest

import oracle
from tests import pyref
from workloads import datagen

E = oracle.EMPTY


def _brute_bq(qcode, codes, d):
    n = codes.shape[0]
    dist = np.array([pyref.distance_by_levels(qcode, codes[v], d) for v in range(n)], dtype=np.int64)
    order = np.lexsort((np.arange(n), dist))  # by (dist, id)
    return order, dist


def _small_case(seed, n=150, d=96, R=6, nq=5):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((n, d)).astype(np.float32)
    q = rng.standard_normal((nq, d)).astype(np.float32)
    adj = datagen.random_regular_graph(n, R, seed + 100, fill=0.9)
    return x, q, adj, oracle.encode(x)


def _hand_graph():
    # Query: 64 coordinates equal to 1.0 -> all signs set, no coordinate above the mean (strict test).
    # A node that differs from the query in a weak coordinate pays 1, in a strong one 2.
    # Wanted distances per node id:
    want = [10, 7, 7, 5, 9, 3, 12, 1]
    codes = np.zeros((8, 2), dtype=np.uint64)
    full = (1 << 64) - 1
    for v, dv in enumerate(want):
        n_strong, n_weak = dv // 2, dv % 2          # flipped coordinates: n_strong strong ones + n_weak weak ones
        flipped = (1 << (n_strong + n_weak)) - 1
        codes[v, 0] = np.uint64(full & ~flipped)
        codes[v, 1] = np.uint64((1 << n_strong) - 1)
    adj = np.array([[1, 2, 6], [3, 4, E], [3, 0, E], [5, E, E], [7, E, E], [3, 1, E], [7, E, E], [E, E, E]],
                   dtype=np.uint32)
    q = np.ones((1, 64), dtype=np.float32)
    return q, codes, adj, want


def test_hand_traced_graph_ef3():
    q, codes, adj, want = _hand_graph()
    for v in range(8):  # the crafted codes do have the wanted distances
        assert oracle.sm_distance(oracle.encode(q)[0], codes[v], 64) == want[v]
    r = oracle.search(q, adj, codes, None, entry=0, k=1, ef=3, visit_cap=8)
    # by hand: expand 0 -> list [(7,1),(7,2),(10,0*)], 6 rejected (12 > 10)
    #          expand 1 -> 3 enters (5), 0 drops; 4 rejected (9 > (7,2))
    #          expand 3 -> 5 enters (3), 2 drops;  expand 5 -> nothing new.  Node 7 (distance 1) is never reached.
    assert r.cand_ids[0].tolist() == [5, 3, 1]
    assert r.cand_dist[0].tolist() == [3, 5, 7]
    assert r.visit_order[0].tolist() == [0, 1, 3, 5, E, E, E, E]
    assert (int(r.n_cand[0]), int(r.n_expanded[0]), int(r.n_dist_evals[0])) == (3, 4, 7)


def test_hand_traced_graph_ef4_tie_broken_by_id():
    q, codes, adj, _ = _hand_graph()
    r = oracle.search(q, adj, codes, None, entry=0, k=1, ef=4, visit_cap=8)
    # ef=4 keeps 4 (9) for a while and node 2 survives: nodes 1 and 2 tie at 7, id 1 goes first both in the
    # expansion order and in the final list.
    assert r.cand_ids[0].tolist() == [5, 3, 1, 2]
    assert r.cand_dist[0].tolist() == [3, 5, 7, 7]
    assert r.visit_order[0].tolist()[:5] == [0, 1, 3, 5, 2]
    assert (int(r.n_expanded[0]), int(r.n_dist_evals[0])) == (5, 7)


def test_exhaustive_ef_equals_brute_force_ranking():
    for seed in (1, 2, 3):
        x, q, adj, codes = _small_case(seed)
        n, d = x.shape
        reach = pyref.bfs_reachable(adj, 0)
        qc = oracle.encode(q)
        r = oracle.search(q, adj, codes, None, entry=0, k=1, ef=n + 5, visit_cap=n)
        for i in range(q.shape[0]):
            order, dist = _brute_bq(qc[i], codes, d)
            order = [int(v) for v in order if int(v) in reach]
            m = int(r.n_cand[i])
            assert m == len(reach) == int(r.n_dist_evals[i])
            assert r.cand_ids[i, :m].tolist() == order
            assert r.cand_dist[i, :m].tolist() == [int(dist[v]) for v in order]
            assert (r.cand_ids[i, m:] == E).all()
            # every reachable node with an out-edge list was expanded exactly once
            vo = r.visit_order[i][r.visit_order[i] != E]
            assert len(vo) == len(set(vo.tolist())) == int(r.n_expanded[i]) == len(reach)


def test_ef1_is_greedy_descent_to_a_local_minimum():
    x, q, adj, codes = _small_case(7, n=300, R=8)
    d = x.shape[1]
    qc = oracle.encode(q)
    r = oracle.search(q, adj, codes, None, entry=3, k=1, ef=1, visit_cap=300)
    for i in range(q.shape[0]):
        path = [int(v) for v in r.visit_order[i] if v != E]
        keys = [(pyref.distance_by_levels(qc[i], codes[v], d), v) for v in path]
        assert path[0] == 3
        assert all(keys[j + 1] < keys[j] for j in range(len(keys) - 1))       # strictly improving
        end = path[-1]
        assert int(r.cand_ids[i, 0]) == end
        for v in adj[end]:
            if v != E:
                assert (pyref.distance_by_levels(qc[i], codes[int(v)], d), int(v)) >= keys[-1]
        # each step moves to the best neighbour of the current node
        for a, b in zip(path[:-1], path[1:]):
            nb = [(pyref.distance_by_levels(qc[i], codes[int(v)], d), int(v)) for v in adj[a] if v != E]
            assert min(nb)[1] == b


def test_invariants_and_row_permutation_invariance():
    x, q, adj, codes = _small_case(21, n=400, d=130, R=10, nq=8)
    d = x.shape[1]
    rng = np.random.default_rng(5)
    adj_perm = adj.copy()
    for u in range(adj.shape[0]):
        adj_perm[u] = adj[u][rng.permutation(adj.shape[1])]
    qc = oracle.encode(q)
    for ef in (1, 4, 17, 64):
        r = oracle.search(q, adj, codes, None, entry=9, k=1, ef=ef, visit_cap=400)
        rp = oracle.search(q, adj_perm, codes, None, entry=9, k=1, ef=ef, visit_cap=400)
        for f in ("cand_ids", "cand_dist", "n_cand", "n_expanded", "n_dist_evals", "visit_order"):
            assert (getattr(r, f) == getattr(rp, f)).all(), f
        for i in range(q.shape[0]):
            m = int(r.n_cand[i])
            assert 1 <= m <= ef
            keys = list(zip(r.cand_dist[i, :m].tolist(), r.cand_ids[i, :m].tolist()))
            assert keys == sorted(keys) and len(set(k[1] for k in keys)) == m
            for dist, v in keys:
                assert dist == pyref.distance_by_levels(qc[i], codes[v], d)
            vo = [int(v) for v in r.visit_order[i] if v != E]
            assert len(vo) == len(set(vo)) == int(r.n_expanded[i])
            # everything in the list was expanded (the search ran to completion)
            assert set(k[1] for k in keys) <= set(vo)
            assert int(r.n_dist_evals[i]) >= m


def test_pool_is_best_ef_of_everything_evaluated():
    # The final list must be the ef smallest keys among all nodes whose distance was computed, i.e. among
    # the out-neighbours of expanded nodes plus the entry.
    x, q, adj, codes = _small_case(33, n=500, d=64, R=8, nq=6)
    qc = oracle.encode(q)
    r = oracle.search(q, adj, codes, None, entry=0, k=1, ef=16, visit_cap=500)
    for i in range(q.shape[0]):
        vo = [int(v) for v in r.visit_order[i] if v != E]
        seen = {0}
        for u in vo:
            seen |= {int(v) for v in adj[u] if v != E}
        assert len(seen) == int(r.n_dist_evals[i])
        keys = sorted((pyref.distance_by_levels(qc[i], codes[v], 64), v) for v in seen)[:16]
        assert [k[1] for k in keys] == r.cand_ids[i, :len(keys)].tolist()


def test_duplicate_and_self_edges_are_harmless():
    x, q, adj, codes = _small_case(41, n=120, R=6)
    adj2 = np.concatenate([adj, adj[:, :2], np.arange(120, dtype=np.uint32)[:, None]], axis=1)
    a = oracle.search(q, adj, codes, None, 0, 1, 12, visit_cap=120)
    b = oracle.search(q, adj2, codes, None, 0, 1, 12, visit_cap=120)
    assert (a.cand_ids == b.cand_ids).all() and (a.visit_order == b.visit_order).all()
    assert (a.n_dist_evals == b.n_dist_evals).all()


def test_threads_do_not_change_results():
    x, q, adj, codes = _small_case(55, n=300, nq=40)
    a = oracle.search(q, adj, codes, x, 0, 5, 20, visit_cap=64, threads=1)
    b = oracle.search(q, adj, codes, x, 0, 5, 20, visit_cap=64, threads=4)
    for f in ("ids", "scores", "cand_ids", "cand_dist", "n_dist_evals", "visit_order"):
        assert (getattr(a, f) == getattr(b, f)).all()


# ---------------------------------------------------------------- Stage 2

def _cos64(q, x):
    q = q.astype(np.float64)
    x = x.astype(np.float64)
    return (x @ q) / (np.linalg.norm(x, axis=1) * np.linalg.norm(q))


def test_rerank_scores_match_numpy_float64():
    x, q, adj, codes = _small_case(61, n=200, d=100, nq=6)
    r = oracle.search(q, adj, codes, x, 0, k=7, ef=24)
    for i in range(q.shape[0]):
        m = int(r.n_cand[i])
        cand = r.cand_ids[i, :m]
        s = _cos64(q[i], x[cand]).astype(np.float32)
        order = np.lexsort((cand, -s))[:7]
        assert r.ids[i].tolist() == cand[order].tolist()
        np.testing.assert_allclose(r.scores[i], s[order], rtol=2e-7, atol=0)
    ids2, sc2, all_sc = oracle.rerank(q, x, r.cand_ids, r.n_cand, 7)
    assert (ids2 == r.ids).all() and (sc2 == r.scores).all()


def test_exhaustive_ef_rerank_is_exact_cosine_knn():
    x, q, adj, codes = _small_case(62, n=180, d=64, R=8, nq=5)
    assert len(pyref.bfs_reachable(adj, 0)) == 180
    r = oracle.search(q, adj, codes, x, 0, k=10, ef=200)
    for i in range(q.shape[0]):
        s = _cos64(q[i], x).astype(np.float32)
        order = np.lexsort((np.arange(180), -s))[:10]
        assert r.ids[i].tolist() == order.tolist()


def test_query_equal_to_a_base_vector_scores_one_and_unit_norm_scores_are_dots():
    w = datagen.scaled("C1", n=300, nq=4)
    x = datagen.make_base(w)
    adj = datagen.random_regular_graph(300, 8, 5)
    codes = oracle.encode(x)
    q = x[[5, 17, 200, 299]]
    r = oracle.search(q, adj, codes, x, 0, k=3, ef=320)
    assert r.ids[:, 0].tolist() == [5, 17, 200, 299]
    np.testing.assert_allclose(r.scores[:, 0], 1.0, atol=1e-7)
    dots = (x[r.ids[0].astype(np.int64)].astype(np.float64) @ q[0].astype(np.float64))
    np.testing.assert_allclose(r.scores[0], dots, atol=1e-6)


def test_short_candidate_list_is_padded_and_zero_norm_scores_zero():
    x = np.zeros((4, 8), dtype=np.float32)
    x[1] = 1.0
    x[2, 0] = -1.0
    adj = np.array([[1, E], [2, E], [3, E], [E, E]], dtype=np.uint32)
    codes = oracle.encode(x)
    q = np.ones((1, 8), dtype=np.float32)
    r = oracle.search(q, adj, codes, x, 0, k=6, ef=6)
    assert int(r.n_cand[0]) == 4
    assert r.ids[0].tolist()[4:] == [E, E] and np.isneginf(r.scores[0, 4:]).all()
    got = dict(zip(r.ids[0, :4].tolist(), r.scores[0, :4].tolist()))
    assert got[1] == pytest.approx(1.0) and got[0] == 0.0 and got[3] == 0.0
    assert got[2] == pytest.approx(-1 / np.sqrt(8))
    assert r.ids[0, :4].tolist() == [1, 0, 3, 2]      # score desc, equal scores by id


def test_bad_arguments_are_rejected():
    x, q, adj, codes = _small_case(70, n=50)
    with pytest.raises(oracle.OracleError):
        oracle.search(q, adj, codes, x, 0, k=9, ef=4)        # k > ef
    with pytest.raises(oracle.OracleError):
        oracle.search(q, adj, codes, x, 50, k=1, ef=4)       # entry out of range
    bad = adj.copy()
    bad[0, 0] = 50
    with pytest.raises(oracle.OracleError):
        oracle.search(q, bad, codes, None, 0, k=1, ef=4)     # edge to a node that does not exist
