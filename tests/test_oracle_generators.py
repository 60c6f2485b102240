"""Pins for the oracle's candidate generators (no GPU): the lattice enumeration against
binomial counts and an independent recursion; the counter-based generator against its
published known-answer vectors and the flat-Dirichlet distribution's closed forms."""
import os
from math import comb

import numpy as np
import pytest
from scipy import stats

from oracle import dirichlet, lattice

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


@pytest.mark.parametrize("m,N", [(1, 5), (2, 7), (3, 10), (4, 6), (5, 4), (3, 1), (6, 3)])
def test_lattice_unrank_matches_recursive_enumeration(m, N):
    total = lattice.count(m, N)
    assert total == comb(N + m - 1, m - 1)
    ref = lattice.compositions(m, N)
    assert ref.shape == (total, m)
    for r in range(total):
        k = lattice.unrank(r, m, N)
        assert list(ref[r]) == k
        assert sum(k) == N and min(k) >= 0
        assert lattice.rank(k, N) == r
    assert list(ref[0]) == [0] * (m - 1) + [N]
    assert list(ref[-1]) == [N] + [0] * (m - 1)
    # consecutive ranks are lexicographic successors
    as_tuples = [tuple(row) for row in ref]
    assert as_tuples == sorted(as_tuples) and len(set(as_tuples)) == total


def test_lattice_config1_count_and_points():
    assert lattice.count(3, 100) == 5151
    X = lattice.points_f32(3, 100)
    assert X.dtype == np.float32 and X.shape == (5151, 3)
    assert np.array_equal(X[0], np.array([0, 0, 1], np.float32))
    assert np.array_equal(X[-1], np.array([1, 0, 0], np.float32))
    assert X[1, 1] == np.float32(1) / np.float32(100)
    with pytest.raises(ValueError):
        lattice.unrank(5151, 3, 100)


def test_lattice_large_rank_arithmetic_is_exact():
    m, N = 12, 60                                   # 3.4e12 points: beyond 32 bits
    total = lattice.count(m, N)
    assert total > 2 ** 40
    for r in (0, 1, total // 3, total - 2, total - 1, 2 ** 33 + 12345):
        k = lattice.unrank(r, m, N)
        assert sum(k) == N and lattice.rank(k, N) == r


def test_philox_known_answers():
    for line in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        w = [int(t, 16) for t in line.split()]
        out = dirichlet.philox4x32_10(np.array(w[0:4], np.uint32), np.array(w[4:6], np.uint32))
        assert [int(v) for v in out] == w[6:10]


def test_dirichlet_rows_are_chunking_invariant_and_on_the_simplex():
    m, seed = 8, 3002
    whole = dirichlet.rows(seed, 0, 1000, m)
    parts = np.concatenate([dirichlet.rows(seed, 0, 333, m), dirichlet.rows(seed, 333, 667, m)])
    assert np.array_equal(whole, parts)
    assert np.all(whole >= 0) and np.allclose(whole.sum(1), 1.0, atol=1e-14)
    u = dirichlet.uniforms(seed, 0, 1000, m)
    assert u.min() > 0 and u.max() <= 1.0
    assert not np.array_equal(whole, dirichlet.rows(seed + 1, 0, 1000, m))
    # 64-bit row indices reach the second counter word
    hi = dirichlet.rows(seed, (1 << 32) + 5, 4, m)
    assert not np.array_equal(hi, dirichlet.rows(seed, 5, 4, m))
    # a width that is not a multiple of four uses a prefix of the same words
    assert np.array_equal(dirichlet.uniforms(seed, 0, 10, 6), dirichlet.uniforms(seed, 0, 10, 8)[:, :6])


@pytest.mark.parametrize("m", [3, 8, 32])
def test_dirichlet_marginals_are_beta(m):
    X = dirichlet.rows(3000 + m, 0, 20000, m)
    # each coordinate of a flat Dirichlet is Beta(1, m-1): mean 1/m,
    # variance (m-1)/(m^2 (m+1)), CDF 1-(1-t)^(m-1)
    assert np.allclose(X.mean(0), 1.0 / m, atol=4 * np.sqrt((m - 1) / (m * m * (m + 1.0)) / 20000))
    assert np.allclose(X.var(0), (m - 1) / (m * m * (m + 1.0)), rtol=0.08)
    for i in (0, m // 2, m - 1):
        ks = stats.kstest(X[:, i], lambda t: 1.0 - (1.0 - t) ** (m - 1))
        assert ks.pvalue > 1e-4
    # coordinates are exchangeable: pairwise covariance -1/(m^2 (m+1))
    cov = np.cov(X[:, 0], X[:, 1])[0, 1]
    var = (m - 1) / (m * m * (m + 1.0))
    assert cov == pytest.approx(-1.0 / (m * m * (m + 1.0)), abs=6 * var / np.sqrt(20000))


def test_lattice_around_exact_rational_cases_and_limits():
    """The shrunk lattice against exact rational arithmetic where every operation is exact in
    float32 (dyadic centre, radius and 1/N), and its two limits."""
    from fractions import Fraction as F
    m, N = 3, 4
    centre = [F(1, 2), F(1, 4), F(1, 4)]
    radius = F(1, 4)
    got = lattice.points_around_f32(m, N, [float(c) for c in centre], float(radius))
    comps = lattice.compositions(m, N)
    assert got.shape == (len(comps), m)
    for row, k in zip(got, comps):
        for i in range(m):
            exact = (1 - radius) * centre[i] + radius * F(int(k[i]), N)
            assert F(float(row[i])) == exact                    # no rounding happened anywhere
        assert sum(F(float(v)) for v in row) == 1
    plain = lattice.points_f32(m, N)
    assert np.array_equal(lattice.points_around_f32(m, N, [0.2, 0.3, 0.5], 1.0), plain)
    rep = lattice.points_around_f32(m, N, [0.2, 0.3, 0.5], 0.0)
    assert np.array_equal(rep, np.tile(np.float32([0.2, 0.3, 0.5]), (len(comps), 1)))
    # generic case: inside the simplex, within radius of the centre (L-infinity), order kept
    c = np.float32([0.1, 0.6, 0.3])
    pts = lattice.points_around_f32(m, 10, c, 0.125)
    assert np.all(pts >= 0) and np.all(np.abs(pts.sum(axis=1) - 1) < 1e-6)
    assert np.all(np.abs(pts - c[None, :]) <= 0.125 + 1e-6)
    assert np.all(np.diff(pts[:, 0]) >= 0)                      # lexicographic order survives the map


def test_dirichlet_around_is_the_affine_image():
    c = np.float32([0.5, 0.25, 0.125, 0.125])
    base = dirichlet.rows(11, 5, 40, 4)
    loc = dirichlet.rows_around(11, 5, 40, 4, c, 0.25)
    assert np.allclose(loc, 0.75 * c[None, :].astype(np.float64) + 0.25 * base, rtol=0, atol=1e-15)
    assert np.allclose(loc.sum(axis=1), 1.0, atol=1e-12)
    assert np.array_equal(dirichlet.rows_around(11, 5, 40, 4, c, 1.0), base)


def test_word_to_uniform_map_by_hand():
    """u = ((w >> 8) + 1) / 2^24: the low eight bits are dropped, the result lies in (0, 1]."""
    w = np.array([0x00000000, 0x000000FF, 0x00000100, 0x7FFFFFFF, 0x80000000, 0xFFFFFF00, 0xFFFFFFFF],
                 dtype=np.uint32)
    u = dirichlet.word_to_uniform(w)
    assert list(u) == [2.0 ** -24, 2.0 ** -24, 2.0 ** -23, 0.5, 0.5 + 2.0 ** -24, 1.0, 1.0]


def test_uniforms_from_the_first_known_answer_vector():
    """Seed 0, row 0, block 0 is the all-zero counter and key of the first published vector, whose
    output words are 6627e8d5 e169c58d bc57ac4c 9b00dbd8.  Dropping the low byte of each and adding
    one gives, by hand, the numerators 6694889, 14772678, 12343213, 10158300 over 2^24."""
    u = dirichlet.uniforms(0, 0, 1, 4)
    assert list(u[0] * 16777216.0) == [6694889.0, 14772678.0, 12343213.0, 10158300.0]
    # m = 3 takes the first three words; m = 5 starts a second block with counter word 2 = 1
    assert list(dirichlet.uniforms(0, 0, 1, 3)[0]) == list(u[0, :3])
    w1 = dirichlet.philox4x32_10(np.array([0, 0, 1, 0], np.uint32), np.array([0, 0], np.uint32))
    assert dirichlet.uniforms(0, 0, 1, 5)[0, 4] == ((int(w1[0]) >> 8) + 1) / 16777216.0


def test_uniforms_counter_and_key_layout():
    """Row index in counter words 0 (low) and 1 (high), block in word 2, word 3 zero; seed low and
    high words as the key: checked through the generator's core, which the published vectors pin."""
    seed, row = 0x0123456789ABCDEF, (7 << 32) + 5
    u = dirichlet.uniforms(seed, row, 2, 12)
    for r in range(2):
        for b in range(3):
            w = dirichlet.philox4x32_10(np.array([(row + r) & 0xFFFFFFFF, (row + r) >> 32, b, 0], np.uint32),
                                        np.array([0x89ABCDEF, 0x01234567], np.uint32))
            assert list(u[r, 4 * b:4 * b + 4]) == [((int(x) >> 8) + 1) / 16777216.0 for x in w]
