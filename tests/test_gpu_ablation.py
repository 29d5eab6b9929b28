"""GPU parity for the two ablation encodings (paper Sec. 5.5, Table 10): 1-bit sign with Hamming distance and the
2-bit uniform quantiser with L1 distance, through encode, distance, scan, beam search and graph construction."""
import numpy as np
import pytest
import torch

import oracle
from tests import util
from workloads import datagen

pytestmark = pytest.mark.gpu
E = util.E
ENCODINGS = [oracle.SIGN1, oracle.SQ2]


@pytest.fixture(scope="module")
def qv():
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2605_02171_amd as m
    assert (m.ENC_SM, m.ENC_SIGN1, m.ENC_SQ2) == (oracle.SM, oracle.SIGN1, oracle.SQ2)
    return m


def _vectors(rng, n, d):
    x = rng.standard_normal((n, d)).astype(np.float32)
    x[0] = 0.0                                    # constant vectors
    x[1] = -3.5
    x[2, ::2] = 0.0                               # zeros and negative zeros among ordinary values
    x[2, 1::4] = -0.0
    x[3] = np.float32(1e-45) * rng.integers(-3, 4, d)     # subnormals only
    x[4] = rng.integers(-2, 3, d)                 # few distinct values: many elements on bucket edges
    x[5] = x[4] * np.float32(2.0 ** 100)
    x[6, : d // 2] = x[6, d // 2: 2 * (d // 2)]   # repeated values
    return x


@pytest.mark.parametrize("enc", ENCODINGS)
@pytest.mark.parametrize("d", [1, 5, 64, 65, 100, 128, 384, 768, 1000, 3072])
def test_encode_bit_exact(qv, enc, d):
    rng = np.random.default_rng(d + enc)
    x = _vectors(rng, 300, d)
    want = oracle.encode(x, threads=8, enc=enc)
    got, status = qv.encode(torch.from_numpy(x).cuda(), want_status=True, enc=enc)
    assert got.shape == want.shape
    assert (qv.to_numpy_u64(got) == want).all()
    assert (qv.to_numpy_u32(status) == 0).all()


@pytest.mark.parametrize("enc", ENCODINGS)
def test_encode_flags_non_finite_input(qv, enc):
    x = np.ones((4, 70), dtype=np.float32)
    x[1, 3], x[3, 69] = np.inf, np.nan
    _, status = qv.encode(torch.from_numpy(x).cuda(), want_status=True, enc=enc)
    assert qv.to_numpy_u32(status).tolist() == [0, 1, 0, 1]


@pytest.mark.parametrize("enc", ENCODINGS)
@pytest.mark.parametrize("d", [3, 64, 200, 768])
def test_distance_bit_exact(qv, enc, d):
    rng = np.random.default_rng(11 * d + enc)
    x = _vectors(rng, 200, d)
    c = oracle.encode(x, enc=enc)
    ia, ib = rng.integers(0, 200, 3000), rng.integers(0, 200, 3000)
    want = oracle.sm_distance_pairs(c, ia, c, ib, d, enc=enc)
    cd = qv.from_numpy_u64(c)
    got = qv.bq_distance(cd, torch.from_numpy(ia).cuda(), cd, torch.from_numpy(ib).cuda(), d, enc=enc)
    assert (qv.to_numpy_u32(got) == want).all()


@pytest.mark.parametrize("enc", ENCODINGS)
@pytest.mark.parametrize("n,d,nq,K", [(4000, 100, 70, 10), (4097, 768, 65, 17), (1500, 64, 64, 64), (2000, 1024, 9, 5)])
def test_scan_bit_exact(qv, enc, n, d, nq, K):
    rng = np.random.default_rng(n + d + K + enc)
    x = rng.standard_normal((n, d)).astype(np.float32)
    x[: n // 3] = x[n // 3: 2 * (n // 3)][: n // 3]       # duplicated vectors: exact distance ties, decided by id
    q = rng.standard_normal((nq, d)).astype(np.float32)
    codes, qc = oracle.encode(x, threads=8, enc=enc), oracle.encode(q, enc=enc)
    want_ids, want_dist = oracle.bq_scan(codes, qc, d, K, threads=8, enc=enc)
    ids, dist = qv.bq_scan(qv.from_numpy_u64(codes), qv.from_numpy_u64(qc), d, K, enc=enc)
    assert (qv.to_numpy_u32(ids) == want_ids).all()
    assert (qv.to_numpy_u32(dist) == want_dist).all()


def _search_both(qv, enc, x, q, adj, entry, k, ef, visit_cap=300):
    codes = oracle.encode(x, threads=8, enc=enc)
    ref = oracle.search(q, adj, codes, x, entry, k, ef, visit_cap=visit_cap, threads=8, enc=enc)
    xd = torch.from_numpy(x).cuda()
    gcodes = qv.encode(xd, enc=enc)
    assert (qv.to_numpy_u64(gcodes) == codes).all()
    index = qv.Index(qv.from_numpy_u32(adj), gcodes, xd, entry, enc=enc)
    for mode in (qv.VISITED_CACHE, qv.VISITED_EXACT):
        index.set_tuning(0, 0, 0, mode)
        out = qv.search(index, torch.from_numpy(q).cuda(), k, ef, trace=True, visit_cap=visit_cap)
        torch.cuda.synchronize()
        assert (qv.to_numpy_u32(out.cand_ids) == ref.cand_ids).all()
        assert (qv.to_numpy_u32(out.cand_dist) == ref.cand_dist).all()
        assert (qv.to_numpy_u32(out.n_cand) == ref.n_cand).all()
        assert (qv.to_numpy_u32(out.n_expanded) == ref.n_expanded).all()
        assert (qv.to_numpy_u32(out.visit_order) == ref.visit_order).all()
        ev, st = qv.to_numpy_u32(out.n_dist_evals), qv.to_numpy_u32(out.status)
        assert (ev >= ref.n_dist_evals).all() and (ev[st == 0] == ref.n_dist_evals[st == 0]).all()
        util.assert_topk_matches(qv.to_numpy_u32(out.ids), out.scores.cpu().numpy(), ref.ids, ref.scores)


@pytest.mark.parametrize("enc", ENCODINGS)
@pytest.mark.parametrize("d,R,ef,k", [(100, 10, 5, 5), (128, 32, 64, 10), (200, 70, 65, 10), (768, 64, 32, 10),
                                      (768, 64, 300, 10), (1024, 64, 64, 10), (130, 130, 600, 7),
                                      # the other widths the kernels are compiled for
                                      (256, 32, 64, 10), (384, 64, 64, 10), (512, 64, 48, 10), (1536, 32, 64, 10),
                                      (2048, 16, 32, 5), (3072, 16, 32, 5)])
def test_search_random_graphs_bit_exact(qv, enc, d, R, ef, k):
    rng = np.random.default_rng(d * 1000 + R + enc)
    n, nq = 3000, 37
    x = rng.standard_normal((n, d)).astype(np.float32)
    q = rng.standard_normal((nq, d)).astype(np.float32)
    adj = datagen.random_regular_graph(n, R, seed=d + R, fill=0.85)
    _search_both(qv, enc, x, q, adj, 5, k, ef, visit_cap=700)


@pytest.mark.parametrize("enc", ENCODINGS)
@pytest.mark.parametrize("lanes", [1, 2, 4, 8, 16])
def test_search_every_gather_width_at_768d(qv, enc, lanes):
    w = datagen.scaled("C2", n=5000, nq=20)
    x, q = datagen.make_base(w), datagen.make_queries(w)
    adj = datagen.random_regular_graph(w.n, 48, seed=lanes)
    codes = oracle.encode(x, threads=8, enc=enc)
    ref = oracle.search(q, adj, codes, x, 3, 10, 48, visit_cap=200, threads=8, enc=enc)
    xd = torch.from_numpy(x).cuda()
    index = qv.Index(qv.from_numpy_u32(adj), qv.encode(xd, enc=enc), xd, 3, enc=enc)
    index.set_tuning(0, lanes, 0, 0)
    out = qv.search(index, torch.from_numpy(q).cuda(), 10, 48, trace=True, visit_cap=200)
    torch.cuda.synchronize()
    assert (qv.to_numpy_u32(out.cand_ids) == ref.cand_ids).all()
    assert (qv.to_numpy_u32(out.cand_dist) == ref.cand_dist).all()
    assert (qv.to_numpy_u32(out.visit_order) == ref.visit_order).all()


def _sorted_rows(adj):
    return np.sort(np.asarray(adj, dtype=np.uint32), axis=1)


@pytest.mark.parametrize("enc", ENCODINGS)
@pytest.mark.parametrize("n,d,R,L,alpha,entry", [(1500, 128, 16, 32, 1.2, 7), (600, 128, 64, 128, 1.2, 11),
                                                 (300, 768, 16, 48, 1.2, 299), (2500, 100, 8, 16, 1.0, 5),
                                                 (800, 300, 16, 32, 1.2, 3), (500, 40, 8, 16, 1.2, 0),
                                                 (400, 384, 16, 32, 1.2, 1), (300, 1024, 16, 32, 1.2, 2),
                                                 (200, 1536, 12, 32, 1.2, 0), (200, 900, 12, 24, 1.2, 5)])
def test_build_matches_oracle(qv, enc, n, d, R, L, alpha, entry):
    rng = np.random.default_rng(n + d + enc)
    x = rng.standard_normal((n, d)).astype(np.float32)
    x[n // 2: n // 2 + 20] = x[:20]              # duplicated vectors: distance ties everywhere
    codes = oracle.encode(x, threads=8, enc=enc)
    util.note(f"ablation construction parity: enc={enc} n={n} d={d} R={R} L={L} (oracle builds first)")
    want = oracle.build_graph(codes, d, R, L, alpha, entry, enc=enc)
    got = qv.build_graph(qv.from_numpy_u64(codes), d, R, L, alpha, entry, enc=enc)
    torch.cuda.synchronize()
    bad = np.nonzero((_sorted_rows(qv.to_numpy_u32(got)) != _sorted_rows(want)).any(axis=1))[0]
    assert bad.size == 0, f"{bad.size} rows differ, first {bad[:5]}"


def test_argument_errors(qv):
    x = torch.ones((4, 64), dtype=torch.float32, device="cuda")
    with pytest.raises(qv.QuiverError) as e:
        qv.encode(x, enc=7)
    assert e.value.code == -1
    codes = torch.zeros((10, 50), dtype=torch.int64, device="cuda")   # 2-bit codes of d = 1600: no construction kernel that wide
    with pytest.raises(qv.QuiverError) as e:
        qv.build_graph(codes, 1600, 8, 16, 1.2, 0, enc=qv.ENC_SQ2)
    assert e.value.code == -9
    assert qv.code_words(768, qv.ENC_SIGN1) == 12 and qv.code_words(768, qv.ENC_SQ2) == 24 and qv.code_words(768, 9) == 0
