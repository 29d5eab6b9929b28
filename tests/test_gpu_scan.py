"""GPU parity for the brute-force code scan and the overlap probe (NEXT row after the search path)."""
import numpy as np
import pytest
import torch

import oracle
from tests import util
from workloads import datagen

pytestmark = pytest.mark.gpu
E = util.E


@pytest.fixture(scope="module")
def qv():
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2605_02171_amd as m
    return m


@pytest.mark.parametrize("n,d,nq,K", [
    (5000, 100, 70, 10), (3000, 200, 1, 16), (4097, 768, 65, 17), (2500, 3072, 30, 10), (1500, 64, 64, 64),
    (7, 128, 5, 10), (1, 64, 3, 1), (20000, 384, 130, 1), (9000, 512, 33, 32),
])
def test_scan_bit_exact(qv, n, d, nq, K):
    rng = np.random.default_rng(n + d + K)
    x = rng.standard_normal((n, d)).astype(np.float32)
    x[: n // 3] = x[n // 3: 2 * (n // 3)][: n // 3]       # duplicated vectors: exact distance ties, decided by id
    q = rng.standard_normal((nq, d)).astype(np.float32)
    codes, qc = oracle.encode(x, threads=8), oracle.encode(q)
    want_ids, want_dist = oracle.bq_scan(codes, qc, d, K, threads=8)
    ids, dist = qv.bq_scan(qv.from_numpy_u64(codes), qv.from_numpy_u64(qc), d, K)
    assert (qv.to_numpy_u32(ids) == want_ids).all()
    assert (qv.to_numpy_u32(dist) == want_dist).all()


def test_scan_of_an_empty_base_set_and_of_no_queries(qv):
    qc = qv.from_numpy_u64(oracle.encode(np.ones((3, 64), dtype=np.float32)))
    none = torch.empty((0, 2), dtype=torch.int64, device="cuda")
    ids, dist = qv.bq_scan(none, qc, 64, 4)
    assert (qv.to_numpy_u32(ids) == E).all() and (qv.to_numpy_u32(dist) == E).all()
    ids, dist = qv.bq_scan(qc, none, 64, 4)
    assert ids.shape == (0, 4)
    with pytest.raises(qv.QuiverError):
        qv.bq_scan(qc, qc, 64, 65)


def test_scan_medium_workload_and_overlap_probe(qv):
    # the paper's probe: on a sample of ~10K vectors, overlap between code-ranked and float32-ranked top 10
    w = datagen.scaled("C2", n=10_000, nq=200)
    x, q = datagen.make_base(w), datagen.make_queries(w)
    codes, qc = oracle.encode(x, threads=8), oracle.encode(q)
    want_ids, want_dist = oracle.bq_scan(codes, qc, w.d, 10, threads=8)
    exact = oracle.cosine_topk(x, q, 10, threads=8)
    xd, qd = torch.from_numpy(x).cuda(), torch.from_numpy(q).cuda()
    ids, dist = qv.bq_scan(qv.encode(xd), qv.encode(qd), w.d, 10)
    assert (qv.to_numpy_u32(ids) == want_ids).all() and (qv.to_numpy_u32(dist) == want_dist).all()
    hits = qv.topk_overlap(ids, qv.from_numpy_u32(exact))
    got = float(qv.to_numpy_u32(hits).sum()) / (200 * 10)
    assert got == oracle.topk_overlap(want_ids, exact)
    per_query = [len(set(a.tolist()) & set(b.tolist())) for a, b in zip(want_ids, exact)]
    assert qv.to_numpy_u32(hits).tolist() == per_query


def test_scan_larger_base_set_sampled(qv):
    # 200k x 768: every returned distance is checked with the oracle, and the whole ranking for a few queries
    w = datagen.scaled("C2", n=200_000, nq=256)
    x, q = datagen.make_base(w), datagen.make_queries(w)
    codes, qc = oracle.encode(x, threads=16), oracle.encode(q)
    ids, dist = qv.bq_scan(qv.from_numpy_u64(codes), qv.from_numpy_u64(qc), w.d, 10)
    ids, dist = qv.to_numpy_u32(ids), qv.to_numpy_u32(dist)
    qi = np.repeat(np.arange(256), 10)
    want = oracle.sm_distance_pairs(qc, qi, codes, ids.reshape(-1).astype(np.int64), w.d)
    assert (want == dist.reshape(-1)).all()
    keys = (dist.astype(np.int64) << 32) | ids
    assert (np.diff(keys, axis=1) > 0).all()
    full_ids, full_dist = oracle.bq_scan(codes, qc[:8], w.d, 10, threads=16)
    assert (ids[:8] == full_ids).all() and (dist[:8] == full_dist).all()
