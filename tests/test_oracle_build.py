"""Pins for the oracle's graph construction (paper Sec. 3.2, Algorithm 1; Sec. 2.2 bidirectional pruning)."""
import numpy as np
import pytest

import oracle
from tests import cases, pyref
from workloads import datagen, graph

E = oracle.EMPTY


def _rows_as_sets(adj):
    return [frozenset(int(v) for v in row if v != E) for row in adj]


def _case(n=700, d=96, seed=1):
    w = datagen.scaled("C1", n=n, nq=20)
    x = datagen.make_base(w) if d == 128 else np.random.default_rng(seed).standard_normal((n, d)).astype(np.float32)
    return x, oracle.encode(x)


def test_tiny_hand_checked_selection():
    # three nodes on a "line" in code space: 0 --1-- 1 --1-- 2 (weak sign flips), d(0,2) = 2.
    # alpha = 1: for node 0 the candidates are 1 (d=1) then 2 (d=2); 2 is dropped because
    # d(2,0)=2 > 1 * d(2,1)=1.  With alpha = 2 it is kept (2 <= 2*1).
    codes = np.array([[0b00, 0], [0b01, 0], [0b11, 0]], dtype=np.uint64)
    strict = oracle.build_graph(codes, 64, 2, 4, 1.0, entry=0)
    relaxed = oracle.build_graph(codes, 64, 2, 4, 2.0, entry=0)
    # node 2 is inserted last: its candidates are 1 (d=1) and 0 (d=2); same rule
    assert _rows_as_sets(strict)[2] == {1}
    assert _rows_as_sets(relaxed)[2] == {0, 1}
    assert _rows_as_sets(strict)[1] >= {0, 2}          # in-edges from both ends reach the middle node


def test_structure_degree_no_self_no_duplicates_reachable():
    x, codes = _case()
    adj = oracle.build_graph(codes, 96, 8, 16, 1.2, entry=3)
    for u, row in enumerate(adj.tolist()):
        ids = [v for v in row if v != E]
        assert len(ids) <= 8 and u not in ids and len(set(ids)) == len(ids) and all(v < 700 for v in ids)
    # in-edges can be pruned away again, so a few nodes may end up unreachable at this small degree
    assert len(pyref.bfs_reachable(adj, 3)) >= 0.9 * 700


def test_matches_the_independent_host_generator_on_the_same_codes():
    # two implementations of the same reading (plain C here, multi-threaded C++ in workloads/) must produce
    # the same neighbour sets
    for n, d, R, L, seed in ((900, 64, 8, 12, 2), (1200, 128, 12, 24, 3), (600, 200, 6, 10, 4)):
        x, codes = _case(n, d, seed)
        a = oracle.build_graph(codes, d, R, L, 1.2, entry=5)
        b = graph.build_graph_from_codes(codes, d, R, L, 1.2, entry=5, threads=4)
        assert _rows_as_sets(a) == _rows_as_sets(b)


def test_batches_change_the_graph_but_not_its_validity():
    x, codes = _case(500, 64, 5)
    seq = oracle.build_graph(codes, 64, 8, 12, 1.2, entry=0, max_batch=1)
    bat = oracle.build_graph(codes, 64, 8, 12, 1.2, entry=0)
    assert _rows_as_sets(seq) != _rows_as_sets(bat)
    for adj in (seq, bat):
        assert len(pyref.bfs_reachable(adj, 0)) >= 0.9 * 500


def test_fully_selected_rows_satisfy_algorithm_1():
    # with batches of one node and R large enough that no row ever overflows, the row of the node inserted
    # last is exactly Algorithm 1 applied to its search result; re-derive it with an independent distance
    x, codes = _case(300, 64, 6)
    n, d, R, L, alpha = 300, 64, 40, 300, 1.2
    adj = oracle.build_graph(codes, d, R, L, alpha, entry=0, max_batch=1)
    t = n - 1
    before = oracle.build_graph(codes[:t], d, R, L, alpha, entry=0, max_batch=1)
    reach = pyref.bfs_reachable(before, 0)
    dist = {v: pyref.distance_by_levels(codes[t], codes[v], d) for v in reach}
    sel = []
    for v in sorted(reach, key=lambda v: (dist[v], v)):
        if all(dist[v] <= alpha * pyref.distance_by_levels(codes[v], codes[s], d) for s in sel):
            sel.append(v)
        if len(sel) == R:
            break
    assert _rows_as_sets(adj)[t] == frozenset(sel)


def test_search_on_the_built_graph_finds_code_space_neighbours():
    w = datagen.scaled("H2", n=3000, nq=30)
    x, q = datagen.make_base(w), datagen.make_queries(w)
    codes, qc = oracle.encode(x), oracle.encode(q)
    adj = oracle.build_graph(codes, w.d, 16, 32, 1.2, entry=0)
    r = oracle.search(q, adj, codes, None, 0, 1, 32)
    ids, _ = oracle.bq_scan(codes, qc, w.d, 10)
    found = np.mean([len(set(a[:10].tolist()) & set(b.tolist())) / 10 for a, b in zip(r.cand_ids, ids)])
    assert found > 0.8


def test_bad_arguments():
    x, codes = _case(50, 64, 7)
    with pytest.raises(oracle.OracleError):
        oracle.build_graph(codes, 64, 4, 8, 0.9, entry=0)
    with pytest.raises(oracle.OracleError):
        oracle.build_graph(codes, 64, 4, 8, 1.2, entry=50)


def _algorithm_1(cands, dist_to_t, code_of, d, R, alpha):
    """Algorithm 1 written out with the level-product distance of tests/pyref (independent of the C oracle)."""
    sel = []
    for c in sorted(cands, key=lambda v: (dist_to_t[v], v)):
        if all(dist_to_t[c] <= alpha * pyref.distance_by_levels(code_of[c], code_of[s], d) for s in sel):
            sel.append(c)
        if len(sel) == R:
            break
    return sel


def test_hub_cap_keeps_the_192_nearest_new_candidates():
    # 196 nodes arrive in one batch and all select the hub (tests/cases.py): 191 "A" nodes at distance 11-12 that
    # are within 4 of each other, then B1..B5 at distance 16, 20, 24, 28, 32.  The hub may consider the 192
    # nearest new candidates by (distance, id) = all A's and B1.  Algorithm 1 then keeps the nearest A (every
    # other A is within 4 of it: 11 > 1.2 * 4), keeps B1, and fills the row from the hub's old neighbours;
    # B2..B5, which Algorithm 1 would keep as well, must not appear.
    d, R, L, alpha = 128, 8, 16, 1.2
    codes, n0, A, B = cases.hub_crowd_codes()
    n = codes.shape[0]
    assert n - n0 == 196 > 192
    adj = oracle.build_graph(codes, d, R, L, alpha, entry=0)
    rows = _rows_as_sets(adj)
    before = _rows_as_sets(oracle.build_graph(codes[:n0], d, R, L, alpha, entry=0))
    for t in range(n0, n):
        assert 0 in rows[t]                          # the hub is every new node's nearest node: always selected
    dist = {v: pyref.distance_by_levels(codes[0], codes[v], d) for v in list(before[0]) + A + B}
    assert sorted(dist[a] for a in A)[0] >= 11 and max(dist[a] for a in A) == 12
    assert [dist[b] for b in B] == [16, 20, 24, 28, 32]
    ranked = sorted(A + B, key=lambda v: (dist[v], v))
    assert ranked[191] == B[0] and ranked[192] == B[1]
    want = _algorithm_1(list(before[0]) + ranked[:192], dist, codes, d, R, alpha)
    assert rows[0] == frozenset(want)
    # what the row must look like, stated directly
    assert len(rows[0] & set(A)) == 1 and ranked[0] in rows[0]
    assert B[0] in rows[0] and not (rows[0] & set(B[1:]))
    assert len(rows[0]) == R and len(rows[0] & before[0]) == R - 2
    # the case is sharp: one candidate more or one fewer gives another row
    for cap in (191, 193):
        other = _algorithm_1(list(before[0]) + ranked[:cap], dist, codes, d, R, alpha)
        assert frozenset(other) != rows[0]
