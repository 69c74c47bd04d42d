"""Pins for the oracle's perturbation stream (CPU only).

The paper only asks for u ~ N(0, I) (Eq. 2); these tests pin the concrete generator to
things other than itself: published Philox known-answer vectors, an fp64 libm Box-Muller
on the same uniforms, scipy's normal distribution, and the Gaussian tail identities of the
appendix lemma on 1-D Gaussian tails."""
import os

import numpy as np
import pytest
from scipy import stats

from oracle import zo_oracle as orc


def test_philox_known_answer_vectors(golden_dir):
    n = 0
    for line in open(os.path.join(golden_dir, "philox4x32_10_kat.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        w = [int(t, 16) for t in line.split()]
        got = orc.philox4x32_10(w[0:4], w[4:6])
        assert [int(v) for v in got] == w[6:10]
        n += 1
    assert n == 3


def test_stream_layout_key_and_counter():
    # word j of the stream = word j&3 of Philox(counter=(blk,0,tensor,0), key=(seed_lo,seed_hi))
    seed, tid = 0x123456789ABCDEF, 37
    words = orc.philox_words(seed, tid, 64)
    for j in (0, 1, 5, 18, 63):
        blk = j >> 2
        ref = orc.philox4x32_10([blk, 0, tid, 0], [seed & 0xFFFFFFFF, seed >> 32])
        assert words[j] == ref[j & 3]


def _box_muller_fp64(word):
    a = word & 0xFFFF
    b = word >> 16
    u1 = (2.0 * a + 1.0) / 131072.0
    theta = 2.0 * np.pi * (b.astype(np.float64) + 0.5) / 65536.0 - np.pi / 4.0
    r = np.sqrt(-2.0 * np.log(u1))
    return r * np.cos(theta), r * np.sin(theta)


def test_normals_match_fp64_box_muller_exhaustive_marginals():
    # every radius input (a) at a few angles, every angle input (b) at a few radii
    worst = 0.0
    for fixed in (0x0000, 0x1234, 0x7FFF, 0x8000, 0xFFFF, 0x4000, 0xC000, 0x3FFF):
        a = np.arange(65536, dtype=np.uint32)
        for words in ((np.uint32(fixed) << 16) | a, (a << 16) | np.uint32(fixed)):
            got = np.array([orc.word_to_normals(w) for w in words[::7]], np.float64)
            c, s = _box_muller_fp64(words[::7].astype(np.uint32))
            worst = max(worst, np.abs(got[:, 0] - c).max(), np.abs(got[:, 1] - s).max())
    # polynomial log / sin / cos + fp32 rounding; |z| <= 4.86
    assert worst < 2e-6, worst


def test_angle_grid_is_uniform_and_quadrants_rotate():
    # b -> b + 0x4000 is a rotation by 90 degrees: (c, s) -> (-s, c), exactly
    for a in (3, 700, 65535):
        for b in (0, 1, 0x1FFF, 0x2000, 0x3FFF):
            c0, s0 = orc.word_to_normals((b << 16) | a)
            c1, s1 = orc.word_to_normals(((b + 0x4000) << 16) | a)
            assert c1 == -s0 and s1 == c0


def test_same_index_same_bits_any_chunking():
    seed, tid = 99, 5
    full = orc.normal(seed, tid, 1000)
    assert np.array_equal(full[123:456], orc.normal(seed, tid, 333, start=123))
    assert full[777] == orc.z_at(seed, tid, 777)
    assert np.array_equal(full, orc.normal(seed, tid, 1000))
    # different tensor id or seed: a different stream
    assert not np.array_equal(full, orc.normal(seed, tid + 1, 1000))
    assert not np.array_equal(full, orc.normal(seed + 1, tid, 1000))
    assert not np.array_equal(full, orc.normal(seed + (1 << 32), tid, 1000))


def test_index_beyond_32_bits():
    # block counter uses both low and high words
    i = (1 << 35) + 3
    blk = i >> 3
    w = orc.philox4x32_10([blk & 0xFFFFFFFF, blk >> 32, 2, 0], [7, 0])
    assert orc.z_at(7, 2, i) == orc.word_to_normals(w[(i >> 1) & 3])[i & 1]


@pytest.fixture(scope="module")
def big_sample():
    return orc.normal(2024, 3, 4_000_000).astype(np.float64)


def test_moments(big_sample):
    z = big_sample
    n = z.size
    assert abs(z.mean()) < 4.0 / np.sqrt(n)
    assert abs(z.var() - 1.0) < 4.0 * np.sqrt(2.0 / n) + 1e-4
    assert abs(stats.skew(z)) < 4.0 * np.sqrt(6.0 / n)
    assert abs(stats.kurtosis(z)) < 4.0 * np.sqrt(24.0 / n) + 1e-3
    assert np.abs(z).max() < 4.86                      # sqrt(2 ln 2^17)


def test_kolmogorov_smirnov(big_sample):
    d, p = stats.kstest(big_sample[:1_000_000], "norm")
    assert p > 1e-3, (d, p)


def test_pairs_uncorrelated(big_sample):
    z = big_sample
    n = z.size // 2
    assert abs(np.mean(z[0::2] * z[1::2])) < 4.0 / np.sqrt(n)
    assert abs(np.mean(z[:-8] * z[8:])) < 4.0 / np.sqrt(z.size)


@pytest.mark.parametrize("t", [0.5, 1.0, 2.0, 3.0])
def test_gaussian_tail_identities(big_sample, t):
    # E|U|1{|U|>=t} = 2 phi(t);  E U^2 1{|U|>=t} = 2(t phi(t) + 1 - Phi(t));  P(|U|>=t) = 2(1 - Phi(t))
    z = big_sample
    n = z.size
    ind = np.abs(z) >= t
    phi, Phi = stats.norm.pdf(t), stats.norm.cdf(t)
    p = 2 * (1 - Phi)
    assert abs(ind.mean() - p) < 4 * np.sqrt(p * (1 - p) / n)
    m1 = (np.abs(z) * ind)
    assert abs(m1.mean() - 2 * phi) < 4 * m1.std() / np.sqrt(n)
    m2 = (z * z * ind)
    assert abs(m2.mean() - 2 * (t * phi + 1 - Phi)) < 4 * m2.std() / np.sqrt(n) + 1e-4
