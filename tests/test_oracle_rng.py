"""Pins of the oracle's random-number layer (Philox words, uniforms, normals).

The Philox round is checked against the same round written with Python's
unbounded integers and against the published known-answer vectors of
Philox4x32-10 (tests/golden/philox4x32_10_kat.txt), the streams against
uniformity / independence statistics.
"""
import os

import numpy as np
from scipy import stats

from oracle import ref

M0, M1 = 0xD2511F53, 0xCD9E8D57
W0, W1 = 0x9E3779B9, 0xBB67AE85
MASK = 0xFFFFFFFF


def philox_bigint(ctr, key, rounds=10):
    c = list(ctr)
    k = list(key)
    for _ in range(rounds):
        p0, p1 = M0 * c[0], M1 * c[2]
        c = [(p1 >> 32) ^ c[1] ^ k[0], p1 & MASK, (p0 >> 32) ^ c[3] ^ k[1], p0 & MASK]
        k = [(k[0] + W0) & MASK, (k[1] + W1) & MASK]
    return c


def test_philox_matches_bigint_rounds():
    rng = np.random.default_rng(1)
    for _ in range(200):
        ctr = [int(x) for x in rng.integers(0, 2**32, 4)]
        key = [int(x) for x in rng.integers(0, 2**32, 2)]
        assert ref.philox(ctr, key) == philox_bigint(ctr, key)
    # extreme operands exercise the 32x32 -> 64 multiply's high word
    assert ref.philox([MASK] * 4, [MASK] * 2) == philox_bigint([MASK] * 4, [MASK] * 2)
    assert ref.philox([0] * 4, [0] * 2) == philox_bigint([0] * 4, [0] * 2)


def test_philox_known_answer_vectors():
    # the generator's published test vectors: a wrong multiplier, Weyl constant, round count or word order fails
    path = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        w = [int(x, 16) for x in r]
        assert ref.philox(w[0:4], w[4:6]) == w[6:10]
        assert philox_bigint(w[0:4], w[4:6]) == w[6:10]
        assert philox_bigint(w[0:4], w[4:6], rounds=9) != w[6:10]


def test_draw_counter_layout():
    seed = 0x0123456789ABCDEF
    got = ref.draw(seed, 5, 7, 11, 2, 3)
    want = ref.philox([5, 7, 11, (2 << 16) | 3], [seed & MASK, seed >> 32])
    assert got == want
    # every field matters
    base = ref.draw(seed, 5, 7, 11, 2, 3)
    for alt in [(6, 7, 11, 2, 3), (5, 8, 11, 2, 3), (5, 7, 12, 2, 3), (5, 7, 11, 1, 3), (5, 7, 11, 2, 4)]:
        assert ref.draw(seed, *alt) != base
    assert ref.draw(seed + 1, 5, 7, 11, 2, 3) != base
    assert ref.draw(seed + (1 << 32), 5, 7, 11, 2, 3) != base


def test_avalanche_one_bit():
    # flipping one counter bit flips about half of the 128 output bits
    flips = []
    for bit in range(0, 128, 7):
        ctr = [0x1234, 0x5678, 0x9ABC, 0xDEF0]
        a = ref.philox(ctr, [1, 2])
        ctr[bit // 32] ^= 1 << (bit % 32)
        b = ref.philox(ctr, [1, 2])
        flips.append(sum(bin(x ^ y).count("1") for x, y in zip(a, b)))
    assert 52 < np.mean(flips) < 76


def test_uniform_is_top_24_bits():
    assert ref.uniform(0) == 0.0
    assert ref.uniform(0xFF) == 0.0
    assert ref.uniform(0x100) == 2.0 ** -24
    assert ref.uniform(MASK) == 1.0 - 2.0 ** -24
    assert ref.uniform(0x80000000) == 0.5
    # exactly representable in float32
    assert float(np.float32(ref.uniform(0xDEADBEEF))) == ref.uniform(0xDEADBEEF)


def test_words_uniformity_chi_square():
    w = ref.words_many(42, 0, 400_000)
    assert len(np.unique(w)) > 399_900  # no structural collisions
    counts = np.bincount(w >> 24, minlength=256)  # top byte
    chi2 = ((counts - len(w) / 256) ** 2 / (len(w) / 256)).sum()
    assert chi2 < stats.chi2.ppf(0.9999, 255)
    counts = np.bincount(w & 0xFF, minlength=256)  # bottom byte
    chi2 = ((counts - len(w) / 256) ** 2 / (len(w) / 256)).sum()
    assert chi2 < stats.chi2.ppf(0.9999, 255)
    # neighbouring counters are uncorrelated
    u = (w >> 8).astype(np.float64) / 2**24
    assert abs(np.corrcoef(u[:-1], u[1:])[0, 1]) < 0.01


def test_normal_pair_formula_and_edges():
    # w0 = 0xFFFFFFFF -> u1 = 1 -> radius 0
    e0, e1 = ref.normal_pair(MASK, 12345)
    assert e0 == 0.0 and e1 == 0.0
    # w0 = 0 -> u1 = 2^-24 (largest radius), angle 0 -> (r, 0)
    e0, e1 = ref.normal_pair(0, 0)
    assert np.isclose(e0, np.sqrt(2 * 24 * np.log(2.0)), rtol=1e-14) and e1 == 0.0
    # quarter turn: u2 = 0.25 -> (0, r)
    e0, e1 = ref.normal_pair(0, 0x40000000)
    assert abs(e0) < 1e-15 * 6 and np.isclose(e1, np.sqrt(2 * 24 * np.log(2.0)), rtol=1e-14)
    # half turn gives (-r, 0)
    e0, e1 = ref.normal_pair(0x7FFFFF00, 0x80000000)
    r = np.sqrt(-2 * np.log((0x7FFFFF + 1) / 2**24))
    assert np.isclose(e0, -r, rtol=1e-14) and abs(e1) < 1e-15


def test_normals_block_layout():
    seed = 99
    n = ref.normals(seed, 3, 0, 17, 2, 17)
    for b in range(5):
        w = ref.draw(seed, 3, 0, 17, 2, b)
        pair0 = ref.normal_pair(w[0], w[1])
        pair1 = ref.normal_pair(w[2], w[3])
        want = [pair0[0], pair0[1], pair1[0], pair1[1]]
        for j in range(4):
            if 4 * b + j < 17:
                assert n[4 * b + j] == want[j]


def test_normal_moments_million():
    x = ref.normals_many(2024, 2, 1_000_000)
    n = len(x)
    assert abs(x.mean()) < 4 / np.sqrt(n)
    assert abs(x.var() - 1) < 4 * np.sqrt(2 / n)
    assert abs((x ** 3).mean()) < 4 * np.sqrt(15 / n)
    assert abs((x ** 4).mean() - 3) < 4 * np.sqrt(96 / n)
    # Kolmogorov-Smirnov against the normal CDF
    assert stats.kstest(x[:200_000], "norm").pvalue > 1e-4
    # the two members of a Box-Muller pair are uncorrelated
    assert abs(np.corrcoef(x[0::2], x[1::2])[0, 1]) < 0.005
