"""Pins for the oracle's two ablation encodings (paper Sec. 5.5 "Encoding Ablation", Table 10):
1-bit sign with Hamming distance and a 2-bit uniform quantiser with L1 distance.

The paper prints no worked example for them, so the pins are hand-worked vectors, reductions to the
Sign-Magnitude functions (which have pins of their own), a second formulation of each distance (popcounts
of whole words / of thermometer planes, written here with numpy), metric properties and brute force."""
import numpy as np
import pytest

import oracle
from oracle import SIGN1, SM, SQ2


def _levels(codes, d):
    W = (d + 63) // 64
    bits = np.array([[(int(c[i // 64]) >> (i % 64)) & 1 for i in range(d)] for c in codes[:, :W]])
    hi = np.array([[(int(c[i // 64]) >> (i % 64)) & 1 for i in range(d)] for c in codes[:, W:]])
    return bits + 2 * hi


def _popcount(a):
    return np.array([bin(int(v)).count("1") for v in a.reshape(-1)]).reshape(a.shape)


def test_code_sizes():
    for d in (1, 64, 65, 768, 1000):
        W = (d + 63) // 64
        assert oracle.code_words(d, SM) == 2 * W and oracle.code_words(d, SQ2) == 2 * W
        assert oracle.code_words(d, SIGN1) == W


def test_sign1_code_is_the_sign_plane_of_the_sign_magnitude_code():
    rng = np.random.default_rng(1)
    for d in (5, 64, 130, 768):
        x = rng.standard_normal((50, d)).astype(np.float32)
        x[0, :3] = [0.0, -0.0, 1e-45]           # zeros are "not positive", the smallest subnormal is
        W = (d + 63) // 64
        assert (oracle.encode(x, enc=SIGN1) == oracle.encode(x)[:, :W]).all()


def test_sign1_distance_is_the_hamming_distance():
    rng = np.random.default_rng(2)
    d = 200
    x = rng.standard_normal((40, d)).astype(np.float32)
    c = oracle.encode(x, enc=SIGN1)
    sm = oracle.encode(x)
    sm[:, 4:] = 0                                # all magnitude bits off: every differing sign costs 1 (Table 1)
    for i in range(0, 40, 3):
        for j in range(0, 40, 7):
            want = int(_popcount(c[i] ^ c[j]).sum())
            assert oracle.distance(c[i], c[j], d, SIGN1) == want
            assert oracle.sm_distance(sm[i], sm[j], d) == want
            assert want == int(((x[i] > 0) != (x[j] > 0)).sum())


def test_sq2_levels_of_hand_worked_vectors():
    # edges at -tau, 0, +tau with tau the mean magnitude (the reading taken for "four equal-width buckets")
    x = np.array([[0.9, -0.1, 0.2, -0.6],       # tau = 0.45
                  [0.5, -0.5, 0.5, -0.5],       # tau = 0.5: an element on an outer edge stays in the inner bucket
                  [0.0, -0.0, 3.0, -1.0],       # tau = 1: zero is "not positive"; -1 sits on the edge -tau
                  [7.0, 7.0, 7.0, 7.0]], dtype=np.float32)
    lv = _levels(oracle.encode(x, enc=SQ2), 4)
    assert lv[0].tolist() == [3, 1, 2, 0]
    assert lv[1].tolist() == [2, 1, 2, 1]
    assert lv[2].tolist() == [1, 1, 3, 1]
    assert lv[3].tolist() == [2, 2, 2, 2]        # constant vector: nothing exceeds the mean


def test_sq2_levels_are_equal_width_buckets_of_the_range_plus_minus_two_tau():
    # away from the edges the level is floor((x + 2 tau) / tau) clamped to 0..3, with tau from exact rationals
    from fractions import Fraction
    rng = np.random.default_rng(3)
    for d in (7, 64, 130):
        x = rng.standard_normal((20, d)).astype(np.float32)
        x[:, 0] *= 8.0                           # beyond the range: outer bucket
        lv = _levels(oracle.encode(x, enc=SQ2), d)
        for r in range(20):
            fr = [Fraction(float(v)) for v in x[r]]
            tau = sum(abs(f) for f in fr) / d
            want = [min(3, max(0, int((f + 2 * tau) // tau))) for f in fr]
            on_edge = [f in (-tau, 0, tau) for f in fr]
            assert not any(on_edge)
            assert lv[r].tolist() == want


def test_sq2_scaling_reflection_and_relation_to_the_sign_magnitude_code():
    rng = np.random.default_rng(4)
    d = 96
    x = rng.standard_normal((30, d)).astype(np.float32)
    c = oracle.encode(x, enc=SQ2)
    assert (oracle.encode(x * 4.0, enc=SQ2) == c).all()
    assert (oracle.encode(x * 0.125, enc=SQ2) == c).all()
    lv, lv_neg = _levels(c, d), _levels(oracle.encode(-x, enc=SQ2), d)
    assert (lv + lv_neg == 3).all()              # mirror image (no zeros in x): bucket b becomes bucket 3 - b
    # the two decisions are those of the method's own code: positive -> upper half, strong -> outer bucket
    sm = oracle.encode(x)
    W = (d + 63) // 64
    pos = np.array([[(int(r[i // 64]) >> (i % 64)) & 1 for i in range(d)] for r in sm[:, :W]])
    strong = np.array([[(int(r[i // 64]) >> (i % 64)) & 1 for i in range(d)] for r in sm[:, W:]])
    assert (lv == np.where(pos == 1, 2 + strong, 1 - strong)).all()
    assert (c[:, W - 1] >> np.uint64(d % 64) == 0).all() and (c[:, 2 * W - 1] >> np.uint64(d % 64) == 0).all()   # padding bits stay zero
    frac = np.bincount(lv.ravel(), minlength=4) / lv.size
    assert abs(frac[0] - frac[3]) < 0.03 and abs(frac[1] - frac[2]) < 0.03 and 0.18 < frac[3] < 0.25   # erfc(1/sqrt(pi))/2 = 0.212


def test_sq2_distance_is_l1_on_levels_and_a_metric():
    rng = np.random.default_rng(4)
    d = 150
    x = rng.standard_normal((25, d)).astype(np.float32)
    c = oracle.encode(x, enc=SQ2)
    lv = _levels(c, d)
    W = (d + 63) // 64
    lo, hi = c[:, :W], c[:, W:]
    t1, t2, t3 = lo | hi, hi, lo & hi            # thermometer planes: level >= 1, >= 2, >= 3
    D = np.zeros((25, 25), dtype=int)
    for i in range(25):
        for j in range(25):
            D[i, j] = oracle.distance(c[i], c[j], d, SQ2)
            assert D[i, j] == int(np.abs(lv[i] - lv[j]).sum())
            assert D[i, j] == int(_popcount(t1[i] ^ t1[j]).sum() + _popcount(t2[i] ^ t2[j]).sum() +
                                  _popcount(t3[i] ^ t3[j]).sum())
    assert (np.diag(D) == 0).all() and (D == D.T).all()
    for k in range(25):
        assert (D <= D[:, [k]] + D[[k], :]).all()   # triangle inequality (L1 is a metric)


def test_distance_pairs_agree_with_single_calls():
    rng = np.random.default_rng(5)
    d = 70
    x = rng.standard_normal((20, d)).astype(np.float32)
    ia, ib = rng.integers(0, 20, 50), rng.integers(0, 20, 50)
    for enc in (SM, SIGN1, SQ2):
        c = oracle.encode(x, enc=enc)
        got = oracle.sm_distance_pairs(c, ia, c, ib, d, enc=enc)
        assert got.tolist() == [oracle.distance(c[a], c[b], d, enc) for a, b in zip(ia, ib)]


@pytest.mark.parametrize("enc", [SIGN1, SQ2])
def test_exhaustive_beam_equals_brute_force_scan(enc):
    # with ef >= n on a connected graph the beam search must return exactly the brute-force ranking
    rng = np.random.default_rng(6 + enc)
    n, d, R = 300, 48, 6
    x = rng.standard_normal((n, d)).astype(np.float32)
    q = rng.standard_normal((7, d)).astype(np.float32)
    adj = np.stack([(np.arange(n) + s) % n for s in (1, 2, 5, 11, 31, 67)], axis=1).astype(np.uint32)
    codes = oracle.encode(x, enc=enc)
    res = oracle.search(q, adj, codes, x, 0, 10, n, enc=enc)
    ids, dist = oracle.bq_scan(codes, oracle.encode(q, enc=enc), d, n, enc=enc)
    assert (res.cand_ids == ids).all() and (res.cand_dist == dist).all()
    qc = oracle.encode(q, enc=enc)
    brute = np.array([[oracle.distance(qc[i], codes[v], d, enc) for v in range(n)] for i in range(7)])
    order = np.lexsort((np.arange(n)[None, :].repeat(7, 0), brute), axis=1)
    assert (ids == order).all()


@pytest.mark.parametrize("enc", [SIGN1, SQ2])
def test_graph_construction_structure(enc):
    rng = np.random.default_rng(20 + enc)
    n, d, R = 400, 64, 8
    x = rng.standard_normal((n, d)).astype(np.float32)
    codes = oracle.encode(x, enc=enc)
    adj = oracle.build_graph(codes, d, R, 16, 1.2, 0, enc=enc)
    for v in range(n):
        row = adj[v][adj[v] != oracle.EMPTY]
        assert len(set(row.tolist())) == len(row) and v not in row and (row < n).all()


def _independent_distance(codes, d, enc):
    """Hamming distance of the sign bits / L1 distance of the levels, from unpacked bits (no oracle call)."""
    if enc == SIGN1:
        W = (d + 63) // 64
        bits = np.array([[(int(c[i // 64]) >> (i % 64)) & 1 for i in range(d)] for c in codes[:, :W]])
        return lambda a, b: int((bits[a] != bits[b]).sum())
    lv = _levels(codes, d)
    return lambda a, b: int(np.abs(lv[a] - lv[b]).sum())


@pytest.mark.parametrize("enc", [SIGN1, SQ2])
def test_last_inserted_row_is_algorithm_1_under_the_encodings_own_distance(enc):
    # batches of one node, L >= n: the node inserted last sees every
    # reachable node as a candidate, and its row is Algorithm 1 over them, sorted by (distance, id), with the
    # alpha test against every neighbour selected so far.  Re-derived here with a distance computed from the
    # unpacked bits.
    rng = np.random.default_rng(30 + enc)
    n, d, R, L, alpha = 260, 64, 40, 260, 1.2
    x = rng.standard_normal((n, d)).astype(np.float32)
    x[200:210] = x[:10]                           # repeated vectors: distance 0 and ties by id
    codes = oracle.encode(x, enc=enc)
    dist = _independent_distance(codes, d, enc)
    adj = oracle.build_graph(codes, d, R, L, alpha, 0, max_batch=1, enc=enc)
    t = n - 1
    before = oracle.build_graph(codes[:t], d, R, L, alpha, 0, max_batch=1, enc=enc)
    seen, frontier = {0}, [0]
    while frontier:
        u = frontier.pop()
        for v in before[u].tolist():
            if v != oracle.EMPTY and v not in seen:
                seen.add(v)
                frontier.append(v)
    sel, rejected = [], 0
    for c in sorted(seen, key=lambda v: (dist(t, v), v)):
        if all(dist(t, c) <= alpha * dist(c, s) for s in sel):
            sel.append(c)
        else:
            rejected += 1
        if len(sel) == R:
            break
    got = set(adj[t][adj[t] != oracle.EMPTY].tolist())
    assert got == set(sel) and len(sel) >= 2 and rejected >= 5    # the alpha test decided, not the degree cap alone
    # and the reverse step: every selected node that had room took t into its own row
    for b in sel:
        if (before[b] != oracle.EMPTY).sum() < R:
            assert t in adj[b].tolist()


def test_more_bits_rank_closer_to_the_exact_ranking():
    # the qualitative finding of Table 10 ("Top-10 overlap" grows from 1-bit sign to 2-bit SM), on low-rank
    # synthetic data of our own; the values themselves are not the paper's
    from workloads import datagen
    w = datagen.scaled("H2", n=4000, nq=40, d=256)
    x, q = datagen.make_base(w), datagen.make_queries(w)
    exact = oracle.cosine_topk(x, q, 10, threads=4)
    overlap = {}
    for enc in (SIGN1, SM, SQ2):
        ids, _ = oracle.bq_scan(oracle.encode(x, enc=enc), oracle.encode(q, enc=enc), w.d, 10, threads=4, enc=enc)
        overlap[enc] = oracle.topk_overlap(ids, exact)
    assert overlap[SIGN1] < overlap[SM]
    assert overlap[SIGN1] < overlap[SQ2]         # Table 10's order: both 2-bit codes rank better than the sign alone
    assert min(overlap.values()) > 0.2
