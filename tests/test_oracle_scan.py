"""Pins for the oracle's brute-force code scan and overlap probe (paper Sec. 6, "Practical compatibility test")."""
import numpy as np

import oracle
from tests import pyref
from workloads import datagen

E = oracle.EMPTY


def _case(seed, n=300, d=100, nq=7):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((n, d)).astype(np.float32)
    q = rng.standard_normal((nq, d)).astype(np.float32)
    return x, q, oracle.encode(x), oracle.encode(q)


def test_scan_equals_sorting_all_distances_of_an_independent_formulation():
    x, q, codes, qc = _case(1)
    ids, dist = oracle.bq_scan(codes, qc, 100, 12)
    for i in range(q.shape[0]):
        dd = np.array([pyref.distance_by_levels(qc[i], codes[v], 100) for v in range(300)])
        order = np.lexsort((np.arange(300), dd))[:12]
        assert ids[i].tolist() == order.tolist() and dist[i].tolist() == dd[order].tolist()


def test_scan_pads_when_fewer_than_k_and_handles_ties_by_id():
    codes = np.zeros((3, 2), dtype=np.uint64)          # three identical codes: all distances tie
    qc = np.array([[5, 0]], dtype=np.uint64)            # two sign bits set, nothing strong
    ids, dist = oracle.bq_scan(codes, qc, 64, 5)
    assert ids[0].tolist() == [0, 1, 2, E, E] and dist[0].tolist() == [2, 2, 2, E, E]


def test_scan_agrees_with_exhaustive_beam_search():
    # two functions of the oracle written separately must rank a connected graph's nodes identically
    x, q, codes, qc = _case(2, n=200, d=64)
    adj = datagen.random_regular_graph(200, 8, 3)
    assert len(pyref.bfs_reachable(adj, 0)) == 200
    r = oracle.search(q, adj, codes, None, 0, 1, 220)
    ids, dist = oracle.bq_scan(codes, qc, 64, 200)
    assert (r.cand_ids[:, :200] == ids).all() and (r.cand_dist[:, :200] == dist).all()


def test_cosine_topk_and_overlap():
    x, q, codes, qc = _case(3, n=250, d=48, nq=9)
    got = oracle.cosine_topk(x, q, 10)
    xn = x.astype(np.float64) / np.linalg.norm(x.astype(np.float64), axis=1, keepdims=True)
    for i in range(9):
        s = (xn @ (q[i].astype(np.float64) / np.linalg.norm(q[i].astype(np.float64)))).astype(np.float32)
        assert got[i].tolist() == np.lexsort((np.arange(250), -s))[:10].tolist()
    a = np.array([[1, 2, 3, 4], [5, 6, E, E]], dtype=np.uint32)
    b = np.array([[4, 3, 9, 8], [6, 5, E, E]], dtype=np.uint32)
    assert oracle.topk_overlap(a, b) == (2 + 2) / 8
    assert oracle.topk_overlap(a, a) == 6 / 8            # padding never counts as a hit


def test_overlap_probe_separates_compatible_from_structureless_data():
    # Sec. 6: the probe is a go/no-go signal; code ranking must track cosine ranking far better on data
    # whose neighbours differ in direction (well-separated points) than on isotropic noise around one centre
    rng = np.random.default_rng(4)
    d = 256
    spread = rng.standard_normal((2000, d)).astype(np.float32)                  # every point its own direction
    tight = (rng.standard_normal((1, d)) + 0.05 * rng.standard_normal((2000, d))).astype(np.float32)
    out = []
    for x in (spread, tight):
        q = x[:50] + 0.3 * rng.standard_normal((50, d)).astype(np.float32) * np.abs(x[:50]).mean()
        ids_bq, _ = oracle.bq_scan(oracle.encode(x), oracle.encode(q), d, 10, threads=4)
        out.append(oracle.topk_overlap(ids_bq, oracle.cosine_topk(x, q, 10, threads=4)))
    assert out[0] > out[1] + 0.1 and out[0] > 0.2
