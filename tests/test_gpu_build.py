"""GPU parity for graph construction in code space (NEXT row): adjacency rows equal the oracle's as sets."""
import numpy as np
import pytest
import torch

import oracle
from tests import cases, util
from workloads import datagen

pytestmark = pytest.mark.gpu
E = util.E


@pytest.fixture(scope="module")
def qv():
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2605_02171_amd as m
    return m


def _sorted_rows(adj):
    a = np.sort(np.asarray(adj, dtype=np.uint32), axis=1)
    return a


def _compare(qv, codes, d, R, L, alpha, entry, max_batch=1 << 20):
    util.note(f"graph construction parity: n={codes.shape[0]} d={d} R={R} L={L} (oracle builds first)")
    want = oracle.build_graph(codes, d, R, L, alpha, entry, max_batch=max_batch)
    got = qv.build_graph(qv.from_numpy_u64(codes), d, R, L, alpha, entry, max_batch=max_batch)
    torch.cuda.synchronize()
    got = qv.to_numpy_u32(got)
    bad = np.nonzero((_sorted_rows(got) != _sorted_rows(want)).any(axis=1))[0]
    assert bad.size == 0, f"{bad.size} rows differ, first {bad[:5]}"
    return got


@pytest.mark.parametrize("n,d,R,L,alpha,entry", [
    (1500, 128, 16, 32, 1.2, 7), (2500, 384, 32, 48, 1.2, 0), (1200, 768, 16, 48, 1.2, 1199),
    (100, 768, 64, 128, 1.2, 0), (600, 128, 64, 128, 1.2, 11), (3000, 100, 8, 16, 1.0, 5),
    (900, 512, 12, 192, 1.5, 450), (300, 1024, 24, 64, 1.2, 3), (40, 128, 64, 64, 1.2, 0),
    # widths the selection kernels are not compiled for (zero-padded in the workspace), and the widest they take
    (700, 300, 16, 32, 1.2, 7), (250, 960, 16, 48, 1.2, 3), (800, 40, 8, 16, 1.2, 0), (800, 200, 16, 32, 1.2, 9),
    (200, 1536, 16, 32, 1.2, 0), (200, 1100, 12, 32, 1.2, 5),
])
def test_build_matches_oracle(qv, n, d, R, L, alpha, entry):
    rng = np.random.default_rng(n + d)
    x = rng.standard_normal((n, d)).astype(np.float32)
    x[n // 2: n // 2 + 20] = x[:20]              # duplicated vectors: distance ties everywhere
    _compare(qv, oracle.encode(x, threads=8), d, R, L, alpha, entry)


def test_build_small_batches_and_single_node(qv):
    rng = np.random.default_rng(3)
    x = rng.standard_normal((600, 128)).astype(np.float32)
    codes = oracle.encode(x)
    _compare(qv, codes, 128, 8, 16, 1.2, 0, max_batch=1)     # strictly sequential insertion
    _compare(qv, codes, 128, 8, 16, 1.2, 0, max_batch=4)
    one = qv.build_graph(qv.from_numpy_u64(codes[:1]), 128, 8, 16, 1.2, 0)
    assert (qv.to_numpy_u32(one) == E).all()


def test_build_hub_takes_only_the_nearest_new_candidates(qv):
    # ~4000 near-copies of node 0 arrive after 10000 ordinary nodes: whole batches of > 192 nodes select the
    # same few hubs, which exercises the cap on new in-edge candidates per batch
    rng = np.random.default_rng(9)
    d = 128
    base = rng.standard_normal((10_000, d)).astype(np.float32)
    crowd = (base[0][None, :] + 0.02 * rng.standard_normal((4_000, d))).astype(np.float32)
    codes = oracle.encode(np.concatenate([base, crowd]), threads=8)
    _compare(qv, codes, d, 8, 16, 1.2, 0)


def test_build_hub_cap_boundary_case(qv):
    # the hand-crafted case of the CPU pin (tests/cases.py): 196 nodes select the hub in one batch, candidate 192 by
    # (distance, id) must be considered and candidate 193 must not
    codes, n0, A, B = cases.hub_crowd_codes()
    got = _compare(qv, codes, 128, 8, 16, 1.2, 0)
    row = set(int(v) for v in got[0] if v != E)
    assert B[0] in row and not (row & set(B[1:])) and len(row & set(A)) == 1


def test_build_then_search_end_to_end(qv):
    # a graph built on the GPU serves the search path like any other input graph: searching it returns, bit for
    # bit, what the oracle returns on the graph the oracle built (the rows are equal as sets and the search does
    # not depend on the order inside a row)
    w = datagen.scaled("H2", n=2_500, nq=100, d=128)
    x, q = datagen.make_base(w), datagen.make_queries(w)
    ocodes = oracle.encode(x, threads=8)
    util.note("end to end: oracle builds 2500 x 128, R=32, L=64")
    oadj = oracle.build_graph(ocodes, w.d, 32, 64, 1.2, 0)
    ref = oracle.search(q, oadj, ocodes, x, 0, 10, 64, threads=8)
    xd = torch.from_numpy(x).cuda()
    codes = qv.encode(xd)
    adj = qv.build_graph(codes, w.d, 32, 64, 1.2, 0)
    index = qv.Index(adj, codes, xd, 0)
    out = qv.search(index, torch.from_numpy(q).cuda(), 10, 64, trace=True)
    torch.cuda.synchronize()
    assert (qv.to_numpy_u32(out.cand_ids) == ref.cand_ids).all()
    assert (qv.to_numpy_u32(out.cand_dist) == ref.cand_dist).all()
    exact = oracle.cosine_topk(x, q, 10, threads=8)
    assert util.recall_at_k(qv.to_numpy_u32(out.ids), exact) > 0.7
    deg = (qv.to_numpy_u32(adj) != E).sum(1)
    assert deg.max() <= 32 and deg.min() >= 1


def test_build_argument_errors(qv):
    codes = torch.zeros((10, 50), dtype=torch.int64, device="cuda")   # d = 1600: planes wider than the selection kernels take
    with pytest.raises(qv.QuiverError) as e:
        qv.build_graph(codes, 1600, 8, 16, 1.2, 0)
    assert e.value.code == -9
    codes = torch.zeros((10, 4), dtype=torch.int64, device="cuda")
    for kw in (dict(R=65), dict(L=193), dict(alpha=0.5), dict(entry=10)):
        args = dict(R=8, L=16, alpha=1.2, entry=0)
        args.update(kw)
        with pytest.raises(qv.QuiverError):
            qv.build_graph(codes, 128, args["R"], args["L"], args["alpha"], args["entry"])
