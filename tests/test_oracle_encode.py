"""Pins for the oracle's 2-bit Sign-Magnitude encoder (paper Sec. 3.1, encoding equations)."""
import math
import os

import numpy as np
import pytest

import oracle
from tests import pyref

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _golden(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                rows.append(line.split())
    return rows


def test_hand_worked_four_dims():
    # x = [0.9, -0.1, 0.2, -0.6]: sum|x| = 1.8, tau = 0.45.
    # pos = [1,0,1,0] -> sign word 0b0101 = 0x5.   |x| > 0.45 -> [1,0,0,1] -> magnitude word 0b1001 = 0x9.
    c = oracle.encode(np.array([[0.9, -0.1, 0.2, -0.6]], dtype=np.float32))
    assert c.shape == (1, 2)
    assert int(c[0, 0]) == 0x5 and int(c[0, 1]) == 0x9


def test_strict_threshold_all_equal_magnitudes():
    # |x_i| = tau for every i: strict ">" leaves the magnitude plane empty.
    c = oracle.encode(np.array([[0.5, -0.5, 0.5, -0.5]], dtype=np.float32))
    assert int(c[0, 0]) == 0x5 and int(c[0, 1]) == 0x0


def test_constant_vector_is_not_strong_despite_rounding():
    # 768 copies of float32(0.1): a float32 running sum does not give exactly 768*x, an exact mean does.
    x = np.full((1, 768), 0.1, dtype=np.float32)
    c = oracle.encode(x)
    assert (c[0, :12] == np.uint64(0xFFFFFFFFFFFFFFFF)).all()
    assert (c[0, 12:] == 0).all()
    # the naive float32 mean would have decided differently for this input (guards the exact reading)
    naive = np.float32(0)
    for v in x[0]:
        naive = np.float32(naive + v)
    assert np.float32(naive / np.float32(768)) != x[0, 0]


def test_zero_and_negative_zero():
    x = np.array([[0.0, -0.0, 0.0, -0.0, 0.0]], dtype=np.float32)
    c = oracle.encode(x)
    assert (c == 0).all()


def test_one_above_mean_by_one_ulp():
    # 63 values v and one value nextafter(v): only the larger one exceeds the exact mean.
    v = np.float32(0.3)
    up = np.nextafter(v, np.float32(1))
    x = np.full((1, 64), v, dtype=np.float32)
    x[0, 17] = up
    c = oracle.encode(x)
    assert int(c[0, 1]) == 1 << 17


def test_wide_dynamic_range_and_denormals_match_exact_rationals():
    rng = np.random.default_rng(5)
    for trial in range(60):
        d = int(rng.integers(1, 200))
        expo = rng.integers(-140, 120, size=d)
        x = (rng.standard_normal(d) * np.exp2(expo.astype(np.float64))).astype(np.float32)
        if trial % 3 == 0:  # put subnormals and zeros in
            x[rng.integers(0, d)] = np.float32(1e-42)
            x[rng.integers(0, d)] = 0.0
        x = np.where(np.isfinite(x), x, np.float32(1.0)).astype(np.float32)
        pos, strong = pyref.encode_exact(x)
        want = pyref.pack(pos, strong)
        got = oracle.encode(x[None, :])[0]
        assert (got == want).all(), f"trial {trial} d={d}"


def test_random_small_vectors_match_exact_rationals():
    rng = np.random.default_rng(11)
    for d in (1, 2, 3, 63, 64, 65, 127, 128, 129, 200):
        x = rng.standard_normal((8, d)).astype(np.float32)
        got = oracle.encode(x)
        for r in range(8):
            pos, strong = pyref.encode_exact(x[r])
            assert (got[r] == pyref.pack(pos, strong)).all()


def test_near_ties_match_exact_rationals():
    # many coordinates sit within a few ulps of the mean
    rng = np.random.default_rng(3)
    for d in (64, 96, 768):
        base = np.float32(0.123456)
        ulps = rng.integers(-3, 4, size=d)
        x = base.view(np.uint32) + ulps.astype(np.int64)
        x = x.astype(np.uint32).view(np.float32)
        x = (x * rng.choice([-1.0, 1.0], size=d)).astype(np.float32)
        pos, strong = pyref.encode_exact(x)
        assert (oracle.encode(x[None, :])[0] == pyref.pack(pos, strong)).all()


def test_padding_bits_are_zero_and_sizes():
    rng = np.random.default_rng(2)
    for d in (1, 5, 63, 65, 100, 130):
        x = np.abs(rng.standard_normal((4, d))).astype(np.float32) + 1.0  # all positive
        c = oracle.encode(x)
        W = (d + 63) // 64
        assert c.shape == (4, 2 * W) and oracle.code_words(d) == 2 * W
        full = (1 << d) - 1
        for r in range(4):
            sign = sum(int(c[r, w]) << (64 * w) for w in range(W))
            mag = sum(int(c[r, W + w]) << (64 * w) for w in range(W))
            assert sign == full          # every real dimension positive, nothing beyond d
            assert mag & ~full == 0


def test_code_size_matches_paper():
    sizes = {k: int(v) for k, v in _golden("sizes.txt")}
    for d in (384, 768):
        nbytes = oracle.code_words(d) * 8
        assert nbytes == d // 4 == sizes[f"code_bytes_per_vector_{d}"]
        assert nbytes * 1_000_000 == sizes[f"signatures_MB_1M_{d}"] * 1_000_000


def test_scale_by_power_of_two_and_negation():
    rng = np.random.default_rng(7)
    x = rng.standard_normal((16, 100)).astype(np.float32)
    c = oracle.encode(x)
    assert (oracle.encode(x * np.float32(8.0)) == c).all()
    assert (oracle.encode(x * np.float32(2.0 ** -20)) == c).all()
    cn = oracle.encode(-x)
    W = 2
    full = [(1 << 64) - 1, (1 << 36) - 1]
    for r in range(16):
        for w in range(W):
            assert int(cn[r, w]) == (~int(c[r, w])) & full[w]     # no zero coordinates here
            assert int(cn[r, W + w]) == int(c[r, W + w])


def test_gaussian_strong_bit_rate_matches_closed_form_and_paper():
    # i.i.d. Gaussian coordinates: tau -> sigma*sqrt(2/pi) (paper Sec. 3.1 footnote), so
    # p_s -> P(|z| > sqrt(2/pi)) = erfc(1/sqrt(pi)) = 0.42494...; Table 13 prints 0.425 for Random-768.
    closed = math.erfc(1.0 / math.sqrt(math.pi))
    printed = {r[0]: float(r[2]) for r in _golden("table13_strong_rate.txt")}["Random-768"]
    assert abs(closed - printed) < 5e-4
    rng = np.random.default_rng(42)
    x = rng.standard_normal((4000, 768)).astype(np.float32)
    c = oracle.encode(x, threads=4)
    bits = np.unpackbits(c.view(np.uint8), axis=1).reshape(4000, 2, 768)
    p_pos = bits[:, 0].mean()
    p_s = bits[:, 1].mean()
    assert abs(p_s - closed) < 2e-3      # 3M bits: sd ~ 3e-4 (plus the finite-D bias of tau)
    assert abs(p_pos - 0.5) < 2e-3


def test_goemans_williamson_on_sign_plane():
    # Theorem 1 / Eq. 1: E[d_H]/D = theta/pi; the text adds Pr[|d_H/D - theta/pi| > 0.05] < 0.044 at D=768.
    rng = np.random.default_rng(9)
    D, n = 768, 3000
    for rho in (0.2, 0.6, 0.9):
        u = rng.standard_normal((n, D))
        v = rho * u + math.sqrt(1 - rho * rho) * rng.standard_normal((n, D))
        cu = oracle.encode(u.astype(np.float32), threads=4)
        cv = oracle.encode(v.astype(np.float32), threads=4)
        x = (cu[:, :12] ^ cv[:, :12]).view(np.uint8)
        dh = np.unpackbits(x, axis=1).sum(axis=1) / D
        cos = np.einsum("ij,ij->i", u, v) / np.linalg.norm(u, axis=1) / np.linalg.norm(v, axis=1)
        theta = np.arccos(cos) / math.pi
        assert abs((dh - theta).mean()) < 2e-3
        assert (np.abs(dh - theta) > 0.05).mean() < 0.044


def test_blind_spot_pair_has_equal_sign_planes_but_distinct_codes():
    # Sec. 2.1: [+0.01,+0.99] and [+0.99,+0.01] share their 1-bit signature; the magnitude bit separates them.
    c = oracle.encode(np.array([[0.01, 0.99], [0.99, 0.01]], dtype=np.float32))
    assert c[0, 0] == c[1, 0] == 3
    assert int(c[0, 1]) == 0b10 and int(c[1, 1]) == 0b01


def test_non_finite_is_rejected():
    for bad in (np.inf, -np.inf, np.nan):
        x = np.ones((2, 8), dtype=np.float32)
        x[1, 3] = bad
        with pytest.raises(oracle.OracleError):
            oracle.encode(x)


def test_threads_do_not_change_codes():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((500, 130)).astype(np.float32)
    assert (oracle.encode(x, threads=1) == oracle.encode(x, threads=4)).all()
