"""Pins for the oracle's symmetric Sign-Magnitude distance (paper Sec. 3.1, Table 1)."""
import os

import numpy as np

import oracle
from tests import pyref

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [l.split() for l in f if l.strip() and not l.startswith("#")]


def _code1(pos, strong):
    return np.array([pos, strong], dtype=np.uint64)  # D = 1: one sign word, one magnitude word


def test_table1_all_sixteen_single_dimension_cases():
    tab = {r[0]: (int(r[1]), int(r[2])) for r in _rows("table1_penalties.txt")}
    for pa in (0, 1):
        for sa in (0, 1):
            for pb in (0, 1):
                for sb in (0, 1):
                    cat = {2: "both_strong", 1: "one_strong_one_weak", 0: "both_weak"}[sa + sb]
                    want = tab[cat][0] if pa == pb else tab[cat][1]
                    assert oracle.sm_distance(_code1(pa, sa), _code1(pb, sb), 1) == want


def test_effective_squared_weight_matches_table13():
    # The paper calls nu_2 = (1+3 p_s)^2 the effective squared weight: for independent magnitude bits with
    # P(strong) = p_s, the mean of (penalty)^2 over the different-sign cases must reproduce the printed nu_2.
    w = {(sa, sb): oracle.sm_distance(_code1(1, sa), _code1(0, sb), 1) for sa in (0, 1) for sb in (0, 1)}
    for name, _d, ps, nu2 in _rows("table13_strong_rate.txt"):
        ps, nu2 = float(ps), float(nu2)
        pr = {0: 1 - ps, 1: ps}
        m2 = sum(pr[sa] * pr[sb] * w[(sa, sb)] ** 2 for sa in (0, 1) for sb in (0, 1))
        # printed p_s has 3 decimals, nu_2 has 2: allow the rounding of both
        assert abs(m2 - nu2) <= 0.005 + 6 * (1 + 3 * ps) * 0.0005, name


def test_hand_worked_pairs():
    enc = lambda v: oracle.encode(np.array([v], dtype=np.float32))[0]
    # x = [0.9,-0.1,0.2,-0.6] (sign 0x5, mag 0x9)  vs  y = [-0.9,-0.1,-0.2,0.6] (sign 0x8, mag 0x9):
    # dim0 differs strong/strong 4; dim1 same 0; dim2 differs weak/weak 1; dim3 differs strong/strong 4.
    x, y = enc([0.9, -0.1, 0.2, -0.6]), enc([-0.9, -0.1, -0.2, 0.6])
    assert (int(y[0]), int(y[1])) == (0x8, 0x9)
    assert oracle.sm_distance(x, y, 4) == 9
    # a = [0.9,0.1] (tau .5: strong,weak) vs b = [-0.4,-0.6] (tau .5: weak,strong): 2 + 2
    assert oracle.sm_distance(enc([0.9, 0.1]), enc([-0.4, -0.6]), 2) == 4
    # the 1-bit blind-spot pair of Sec. 2.1 agrees in sign everywhere: distance 0 although the codes differ
    assert oracle.sm_distance(enc([0.01, 0.99]), enc([0.99, 0.01]), 2) == 0


def _random_codes(rng, n, d):
    W = (d + 63) // 64
    c = rng.integers(0, 2 ** 64, size=(n, 2 * W), dtype=np.uint64)
    if d % 64:
        mask = np.uint64((1 << (d % 64)) - 1)
        c[:, W - 1] &= mask
        c[:, 2 * W - 1] &= mask
    return c


def test_identity_symmetry_range():
    rng = np.random.default_rng(0)
    for d in (1, 37, 64, 100, 768):
        c = _random_codes(rng, 40, d)
        for i in range(0, 40, 2):
            a, b = c[i], c[i + 1]
            dab = oracle.sm_distance(a, b, d)
            assert oracle.sm_distance(a, a, d) == 0
            assert dab == oracle.sm_distance(b, a, d)
            assert 0 <= dab <= 4 * d


def test_antipodal_distance_closed_form():
    # d(x, -x) = sum_i (1+strong_i)^2 = D + 3 * #strong when no coordinate is zero
    rng = np.random.default_rng(4)
    x = rng.standard_normal((10, 200)).astype(np.float32)
    c, cn = oracle.encode(x), oracle.encode(-x)
    for r in range(10):
        n_strong = sum(pyref.unpack(c[r], 200)[1])
        assert oracle.sm_distance(c[r], cn[r], 200) == 200 + 3 * n_strong


def test_equals_signed_level_inner_product_form():
    # independent formulation: levels l = 1 + strong, signed a = +-l: d = (<|a|,|b|> - <a,b>) / 2
    rng = np.random.default_rng(8)
    for d in (3, 64, 65, 130, 384):
        c = _random_codes(rng, 30, d)
        for i in range(0, 30, 2):
            assert oracle.sm_distance(c[i], c[i + 1], d) == pyref.distance_by_levels(c[i], c[i + 1], d)


def test_word_level_popcount_forms_agree_with_lookup():
    rng = np.random.default_rng(12)
    for d in (64, 128, 768):
        c = _random_codes(rng, 20, d)
        for i in range(0, 20, 2):
            f1, f2 = pyref.popcount_forms(c[i], c[i + 1], d)
            assert f1 == f2 == oracle.sm_distance(c[i], c[i + 1], d)


def test_padding_contributes_nothing():
    rng = np.random.default_rng(13)
    x = rng.standard_normal((6, 70)).astype(np.float32)
    c70 = oracle.encode(x)
    # the same numbers as the first 70 of 128 dims, the rest zero: zero coords are (pos 0, strong 0) on both
    # sides and agree in sign, so they add nothing -- but the mean changes, so compare with level arithmetic
    xp = np.zeros((6, 128), dtype=np.float32)
    xp[:, :70] = x
    c128 = oracle.encode(xp)
    for i in range(0, 6, 2):
        assert oracle.sm_distance(c128[i], c128[i + 1], 128) == pyref.distance_by_levels(c128[i], c128[i + 1], 128)
        assert oracle.sm_distance(c70[i], c70[i + 1], 70) == pyref.distance_by_levels(c70[i], c70[i + 1], 70)


def test_pairs_entry_point():
    rng = np.random.default_rng(14)
    d = 200
    a, b = _random_codes(rng, 50, d), _random_codes(rng, 60, d)
    ia = rng.integers(0, 50, size=300)
    ib = rng.integers(0, 60, size=300)
    out = oracle.sm_distance_pairs(a, ia, b, ib, d)
    for p in range(0, 300, 7):
        assert out[p] == pyref.distance_by_levels(a[ia[p]], b[ib[p]], d)


def test_sign_plane_gives_a_lower_bound_of_the_distance():
    # Table 1: a dimension with differing signs costs (1 + strong_a)(1 + strong_b) >= (1 + strong_a).  So the distance
    # with b's magnitude bits taken as zero -- all of them, or all but a known prefix -- never exceeds the distance,
    # and equals it when every magnitude bit is known.  (The library's split code layout reads b's magnitude words
    # only where this bound does not already decide.)
    rng = np.random.default_rng(21)
    d = 200
    W = (d + 63) // 64
    x = rng.standard_normal((40, d)).astype(np.float32)
    c = oracle.encode(x)
    for i in range(0, 40, 3):
        for j in range(1, 40, 4):
            full = oracle.sm_distance(c[i], c[j], d)
            assert full == pyref.distance_by_levels(c[i], c[j], d)
            previous = -1
            for known in range(W + 1):                      # magnitude words of b that are known
                masked = c[j].copy()
                masked[W + known:] = 0
                bound = oracle.sm_distance(c[i], masked, d)
                assert previous <= bound <= full            # more known words never loosen the bound
                previous = bound
            assert previous == full
