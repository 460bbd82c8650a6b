"""Pins for the oracle's random-number layer (Philox4x32-10, uniforms, normals, draw keys)."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
from scipy import stats

from oracle import nuts_ref as R

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")
M32 = 0xFFFFFFFF


def philox_bigint(ctr, key, rounds=10):
    """Philox4x32 written from the round definition of Salmon et al. (SC'11, Section 3.3)
    with Python integers; shares nothing with the C code."""
    c = [int(x) & M32 for x in ctr]
    k = [int(x) & M32 for x in key]
    for _ in range(rounds):
        p0 = 0xD2511F53 * c[0]
        p1 = 0xCD9E8D57 * c[2]
        c = [((p1 >> 32) ^ c[1] ^ k[0]) & M32, p1 & M32, ((p0 >> 32) ^ c[3] ^ k[1]) & M32, p0 & M32]
        k = [(k[0] + 0x9E3779B9) & M32, (k[1] + 0xBB67AE85) & M32]
    return c


def test_known_answers():
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    assert len(rows) >= 2
    for row in rows:
        v = [int(x, 16) for x in row]
        assert list(R.philox(v[0:4], v[4:6])) == v[6:10]
        assert philox_bigint(v[0:4], v[4:6]) == v[6:10]


def test_c_equals_bigint_on_random_inputs():
    rng = np.random.default_rng(7)
    words = rng.integers(0, 2**32, size=(10000, 6), dtype=np.uint64)
    for w in words:
        assert list(R.philox(w[:4], w[4:])) == philox_bigint(w[:4], w[4:])


def test_is_a_bijection_on_a_counter_slice():
    outs = {tuple(R.philox([i, 5, 6, 7], [11, 13])) for i in range(4096)}
    assert len(outs) == 4096


def test_draw_counter_layout():
    seed = 0x0123456789ABCDEF
    for (index, tag, level, it, chain) in [(0, 0, 0, 0, 0), (3, 1, 0, 17, 4095), (1023, 3, 9, 999, 16383),
                                           (7, 4, 0, 2**31, 2**32 - 1)]:
        want = philox_bigint([index, tag | (level << 8), it, chain], [seed & M32, seed >> 32])
        assert list(R.draw(seed, index, tag, level, it, chain)) == want


def test_uniform_is_exact_cell_midpoint():
    rng = np.random.default_rng(3)
    cases = [(0, 0), (M32, M32), (0, M32), (M32, 0), (63, 63), (64, 64)] + [tuple(x) for x in
                                                                          rng.integers(0, 2**32, size=(2000, 2))]
    for a, b in cases:
        a, b = int(a), int(b)
        m = ((a >> 6) << 26) | (b >> 6)
        want = Fraction(2 * m + 1, 2**53)
        got = R.uniform(a, b)
        assert Fraction(got) == want
        assert 0.0 < got < 1.0
    assert R.uniform(0, 0) == 2.0**-53
    assert R.uniform(M32, M32) == 1.0 - 2.0**-53


def test_normal_pair_is_box_muller():
    rng = np.random.default_rng(5)
    for w in rng.integers(0, 2**32, size=(500, 4)):
        u1 = Fraction(2 * (((int(w[0]) >> 6) << 26) | (int(w[1]) >> 6)) + 1, 2**53)
        u2 = Fraction(2 * (((int(w[2]) >> 6) << 26) | (int(w[3]) >> 6)) + 1, 2**53)
        rho = math.sqrt(-2.0 * math.log(float(u1)))
        z0, z1 = R.normal_pair(w)
        assert z0 == pytest.approx(rho * math.cos(2 * math.pi * float(u2)), rel=1e-13, abs=1e-15)
        assert z1 == pytest.approx(rho * math.sin(2 * math.pi * float(u2)), rel=1e-13, abs=1e-15)
        assert z0 * z0 + z1 * z1 == pytest.approx(rho * rho, rel=1e-13)


def test_normals_and_uniforms_have_the_right_distribution():
    n = 100000
    z = np.empty(2 * n)
    u = np.empty(2 * n)
    for i in range(n):
        w = R.draw(99, i, R.TAG_MOMENTUM, 0, 3, 5)
        z[2 * i], z[2 * i + 1] = R.normal_pair(w)
        u[2 * i], u[2 * i + 1] = R.uniform(w[0], w[1]), R.uniform(w[2], w[3])
    assert stats.kstest(z, "norm").pvalue > 1e-3
    assert stats.kstest(u, "uniform").pvalue > 1e-3
    assert abs(z.mean()) < 5 / math.sqrt(2 * n)
    assert abs(z.var() - 1) < 5 * math.sqrt(2 / (2 * n))
    assert abs(np.mean(z**4) - 3) < 5 * math.sqrt(96 / (2 * n))
    assert abs(np.corrcoef(z[0::2], z[1::2])[0, 1]) < 5 / math.sqrt(n)
    # neighbouring counters are unrelated
    assert abs(np.corrcoef(z[0:-2:2], z[2::2])[0, 1]) < 5 / math.sqrt(n)


def test_direction_bit_is_fair():
    bits = np.array([R.draw(1, j, R.TAG_DIRECTION, 0, t, 0)[0] >> 31 for j in range(10) for t in range(2000)])
    assert abs(bits.mean() - 0.5) < 5 * 0.5 / math.sqrt(bits.size)


def test_logaddexp():
    rng = np.random.default_rng(1)
    for a, b in rng.normal(scale=50, size=(2000, 2)):
        assert R.logaddexp(a, b) == pytest.approx(np.logaddexp(a, b), rel=1e-15, abs=1e-15)
    ninf = -math.inf
    assert R.logaddexp(ninf, ninf) == ninf
    assert R.logaddexp(ninf, 1.5) == 1.5
    assert R.logaddexp(2.5, ninf) == 2.5
    assert R.logaddexp(0.0, 0.0) == pytest.approx(math.log(2.0), rel=1e-16)
