"""Pins for the oracle's counter-based gradient noise (Assumption 2: zero mean, bounded variance).

The generator is this build's choice (the paper only fixes the moments); what pins it is the
published Philox known answers, libm for the two transcendental pieces, and the textbook
distributions it must reproduce.
"""
import math
import os

import numpy as np
import pytest
from scipy import stats

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def test_philox_known_answers(oracle_mod):
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        w = [int(x, 16) for x in r]
        out = oracle_mod.philox4x32_10(w[0:4], w[4:6])
        assert out.tolist() == w[6:10]


def test_philox_counter_words_are_not_interchangeable(oracle_mod):
    base = oracle_mod.philox4x32_10([1, 2, 3, 4], [5, 6]).tolist()
    seen = {tuple(base)}
    for ctr, key in [([2, 1, 3, 4], [5, 6]), ([1, 2, 4, 3], [5, 6]), ([1, 2, 3, 4], [6, 5]),
                     ([1, 3, 2, 4], [5, 6])]:
        seen.add(tuple(oracle_mod.philox4x32_10(ctr, key).tolist()))
    assert len(seen) == 5


def _words(rng, m):
    w = rng.integers(0, 1 << 32, size=m, dtype=np.uint64)
    edge = np.array([0, 0xFF, 0x100, 0xFFFFFFFF, 0xFFFFFF00, 0x80000000, 0x7FFFFFFF,
                     0x3504F300, 0x3504F400, 0xB504F300, 0x20000000, 0x1FFFFF00, 0xDFFFFF00,
                     0xE0000000, 0x5FFFFF00, 0x60000000, 0x9FFFFF00, 0xA0000000], dtype=np.uint64)
    return np.concatenate([edge, w])


def test_neg2ln_matches_libm(oracle_mod):
    rng = np.random.default_rng(11)
    for w in _words(rng, 20000):
        w = int(w)
        u = ((w >> 8) + 1) / 2.0 ** 24
        want = -2.0 * math.log(u)
        got = oracle_mod.neg2ln_uniform(w)
        assert got >= 0.0
        assert abs(got - want) <= 2e-6 * max(1.0, want), (hex(w), got, want)
    assert oracle_mod.neg2ln_uniform(0xFFFFFFFF) == 0.0          # u = 1 exactly


def test_unit_circle_matches_libm(oracle_mod):
    rng = np.random.default_rng(12)
    for w in _words(rng, 20000):
        w = int(w)
        ang = 2.0 * math.pi * ((w >> 8) + 0.5) / 2.0 ** 24
        c, s = oracle_mod.unit_circle_point(w)
        assert abs(c - math.cos(ang)) <= 3e-7, hex(w)
        assert abs(s - math.sin(ang)) <= 3e-7, hex(w)


def test_unit_circle_angles_sit_in_the_middle_of_their_steps(oracle_mod):
    """The 2^24 angles are 2 pi (a + 1/2) / 2^24: none lies on an axis, and the set is its own mirror
    image, a and 2^24 - 1 - a giving the same cosine and opposite sines bit for bit (the offset
    inside the quadrant changes sign exactly).  The first angle is pi / 2^24, whose sine in fp32 is
    the angle itself."""
    c, s = oracle_mod.unit_circle_point(0)
    assert s == float(np.float32(math.pi / 2.0 ** 24)) and c == 1.0
    rng = np.random.default_rng(13)
    for a in [0, 1, 0x1FFFFF, 0x200000, 0x3FFFFF, 0x400000, 0x7FFFFF, 0x800000] + [int(v) for v in rng.integers(0, 1 << 24, 3000)]:
        c1, s1 = oracle_mod.unit_circle_point(a << 8)
        c2, s2 = oracle_mod.unit_circle_point(((1 << 24) - 1 - a) << 8)
        assert c1 == c2 and s1 == -s2 and s1 != 0.0 and c1 != 0.0, hex(a)


def test_draws_are_box_muller_of_the_philox_words(oracle_mod):
    seed, t, worker = 0x1234567855AA33CC, (7 << 32) | 9, 3
    key = [seed & 0xFFFFFFFF, seed >> 32]

    def radius_sq(word):
        return -2.0 * math.log(((int(word) >> 8) + 1) / 2.0 ** 24)

    def angle(word):
        return 2.0 * math.pi * ((int(word) >> 8) + 0.5) / 2.0 ** 24

    for j in [0, 1, 2, 3, 76, 77, 78, 79, 2 ** 31 + 5, 2 ** 31 + 6]:
        # normal: the block of counter (j >> 2, worker, t_lo, t_hi) serves four coordinates with
        # the Box-Muller pairs of its words (0, 1) and (2, 3): z = sqrt(-2 ln u) (cos | sin)(2 pi v)
        w = oracle_mod.philox4x32_10([j >> 2, worker, t & 0xFFFFFFFF, t >> 32], key)
        pair = (j >> 1) & 1
        r, ang = math.sqrt(radius_sq(w[2 * pair])), angle(w[2 * pair + 1])
        want = r * (math.sin(ang) if j & 1 else math.cos(ang))
        got = oracle_mod.noise_z(seed, t, worker, j, 1)
        assert abs(got - want) <= 5e-6 * max(1.0, abs(want)), j
        # Student-t(3): three words to a coordinate, taken in order from the twelve words of the
        # blocks with counters (3q, ..), (3q+1, ..), (3q+2, ..), q = j >> 2: z0 over the root of a
        # chi-square(3)/3 built from the pair's second normal and the squared radius -2 ln u of
        # the third word
        twelve = []
        for b in range(3):
            twelve += list(oracle_mod.philox4x32_10([3 * (j >> 2) + b, worker, t & 0xFFFFFFFF, t >> 32], key))
        w = twelve[3 * (j & 3):3 * (j & 3) + 3]
        r, ang = math.sqrt(radius_sq(w[0])), angle(w[1])
        z0, z1 = r * math.cos(ang), r * math.sin(ang)
        want_t = z0 / math.sqrt((z1 * z1 + radius_sq(w[2])) / 3.0)
        got_t = oracle_mod.noise_z(seed, t, worker, j, 2)
        assert abs(got_t - want_t) <= 2e-5 * max(1.0, abs(want_t)), j
    assert oracle_mod.noise_z(seed, t, worker, 5, 0) == 0.0


def test_the_four_t3_draws_of_a_quad_are_uncorrelated(oracle_mod):
    z = oracle_mod.noise_fill(4, 22, 0, 0, 400_000, 2).astype(np.float64).reshape(-1, 4)
    # t(3) has no finite fourth moment: compare ranks (Spearman) of the values and of their magnitudes
    for cols in (z, np.abs(z)):
        rho = stats.spearmanr(cols).statistic
        assert np.abs(rho - np.eye(4)).max() < 1e-2


def test_the_four_normals_of_a_block_are_uncorrelated(oracle_mod):
    z = oracle_mod.noise_fill(3, 21, 1, 0, 400_000, 1).astype(np.float64).reshape(-1, 4)
    corr = np.corrcoef(z.T)
    assert np.abs(corr - np.eye(4)).max() < 1e-2
    # and so are their squares (cos and sin of one angle are dependent; times an independent
    # Rayleigh radius they are independent normals)
    corr2 = np.corrcoef((z * z).T)
    assert np.abs(corr2 - np.eye(4)).max() < 1e-2


def test_normal_distribution(oracle_mod):
    z = oracle_mod.noise_fill(0, 3, 1, 0, 400_000, 1).astype(np.float64)
    assert abs(z.mean()) < 5e-3
    assert abs(z.var() - 1.0) < 1e-2
    assert abs(stats.skew(z)) < 2e-2
    assert abs(stats.kurtosis(z)) < 5e-2
    assert stats.kstest(z, "norm").pvalue > 1e-3
    # tails: P(|z| > 3) = 2.6998e-3
    assert abs((np.abs(z) > 3).mean() - 2.6998e-3) < 4e-4


def test_student_t3_distribution(oracle_mod):
    z = oracle_mod.noise_fill(2, 9, 0, 0, 400_000, 2).astype(np.float64)
    assert abs(np.median(z)) < 5e-3
    assert stats.kstest(z, "t", args=(3,)).pvalue > 1e-3
    # heavy tail: P(|t3| > 5) = 2 * sf(5)
    want = 2 * stats.t.sf(5.0, 3)
    assert abs((np.abs(z) > 5).mean() - want) < 1e-3
    assert np.abs(z).max() > 30.0


def test_draws_depend_on_every_coordinate(oracle_mod):
    a = oracle_mod.noise_fill(5, 10, 2, 0, 1000, 1)
    assert np.array_equal(a, oracle_mod.noise_fill(5, 10, 2, 0, 1000, 1))
    for other in (oracle_mod.noise_fill(6, 10, 2, 0, 1000, 1),
                  oracle_mod.noise_fill(5, 11, 2, 0, 1000, 1),
                  oracle_mod.noise_fill(5, 10, 3, 0, 1000, 1),
                  oracle_mod.noise_fill(5, 10, 2, 1, 1000, 1)):
        assert abs(np.corrcoef(a, other)[0, 1]) < 0.15
    # the fill is the per-element function evaluated at consecutive j
    assert a[17] == np.float32(oracle_mod.noise_z(5, 10, 2, 17, 1))
    # workers are uncorrelated at the same (t, j): the noise is per worker
    b = oracle_mod.noise_fill(5, 10, 3, 0, 200_000, 1)
    c = oracle_mod.noise_fill(5, 10, 2, 0, 200_000, 1)
    assert abs(np.corrcoef(b, c)[0, 1]) < 1e-2
