"""Pins for the oracle's random-number layer: Philox4x32-10, the uniform and
Gaussian transforms, the shared-vector fills and the peer permutation.

Nothing here touches the GPU.  Each test ties the C oracle to something other
than itself: published known-answer vectors, numpy's Philox (same round
structure at 64-bit width), a pure-Python big-integer restatement, exact
rational arithmetic, or distributional facts.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
from scipy import stats as sst

import brute

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def _kat_rows():
    rows = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            w = [int(t, 16) for t in line.split()]
            rows.append((w[0:4], w[4:6], w[6:10]))
    return rows


def test_philox_known_answers(oracle):
    rows = _kat_rows()
    assert len(rows) == 3
    for ctr, key, out in rows:
        assert list(oracle.philox4x32_10(ctr, key)) == out
        assert list(brute.philox4(ctr, key, 32)) == out


def test_philox_round_structure_matches_numpy_at_64_bits():
    """numpy ships Philox-4x64-10; the same generic round code, with the
    64-bit constants, must reproduce it.  numpy bumps the counter once before
    its first block, hence the +1."""
    rng = np.random.default_rng(7)
    for _ in range(50):
        ctr = [int(w) for w in rng.integers(0, 2**63, 4)]
        key = [int(w) for w in rng.integers(0, 2**63, 2)]
        got = [int(w) for w in np.random.Philox(counter=ctr, key=key).random_raw(4)]
        bumped = [ctr[0] + 1] + ctr[1:]
        assert got == list(brute.philox4(bumped, key, 64))


def test_philox_oracle_equals_bigint_restatement(oracle):
    rng = np.random.default_rng(11)
    for _ in range(5000):
        ctr = [int(w) for w in rng.integers(0, 2**32, 4)]
        key = [int(w) for w in rng.integers(0, 2**32, 2)]
        assert oracle.philox4x32_10(ctr, key) == brute.philox4(ctr, key, 32)
    # structured corners: single set bits in every input word
    for word in range(6):
        for bit in (0, 15, 31):
            w = [0] * 6
            w[word] = 1 << bit
            assert oracle.philox4x32_10(w[:4], w[4:]) == brute.philox4(w[:4], w[4:], 32)


def test_philox_output_bytes_look_uniform(oracle):
    words = []
    for q in range(4096):
        words.extend(oracle.philox4x32_10((q, 3, 9, 0), (0x61104581, 0x1)))
    b = np.array(words, dtype=np.uint32).view(np.uint8)
    counts = np.bincount(b, minlength=256)
    chi2 = ((counts - b.size / 256) ** 2 / (b.size / 256)).sum()
    assert sst.chi2.sf(chi2, 255) > 1e-4


def test_u01_is_exact_open_and_symmetric(oracle):
    for r in [0, 1, 511, 512, 2**31 - 1, 2**31, 2**32 - 512, 2**32 - 1, 0x12345678, 0xDEADBEEF]:
        u = oracle.u01(r)
        assert Fraction(float(u)) == brute.u01_fraction(r)
        assert 0.0 < float(u) < 1.0
        assert Fraction(float(u)) + Fraction(float(oracle.u01(r ^ 0xFFFFFFFF))) == 1
    assert float(oracle.u01(0)) == 2.0 ** -24
    assert float(oracle.u01(2**32 - 1)) == 1.0 - 2.0 ** -24


def test_uniform_noise_matches_exact_rational_rounding(oracle):
    rng = np.random.default_rng(3)
    for _ in range(300):
        words = [int(w) for w in rng.integers(0, 2**32, 4)]
        got = oracle.noise4(words, 1)
        for m in range(4):
            assert Fraction(float(got[m])) == brute.uniform_noise_exact(words[m])


def _noise_samples(oracle, kind, n_quads, replica=0, step=0):
    out = np.empty((n_quads, 4), np.float32)
    for q in range(n_quads):
        out[q] = oracle.noise4(brute.philox4((q, replica, step, 0), (0x61104581, 0x1)), kind)
    return out


def test_uniform_noise_moments(oracle):
    z = _noise_samples(oracle, 1, 20000).astype(np.float64).ravel()
    n = z.size
    assert abs(z.mean()) < 4 / math.sqrt(n)
    assert abs(z.var() - 1.0) < 0.02
    assert abs(((z - z.mean()) ** 4).mean() / z.var() ** 2 - 1.8) < 0.03
    assert np.abs(z).max() < math.sqrt(3.0)


def test_gaussian_noise_is_standard_normal(oracle):
    z4 = _noise_samples(oracle, 0, 25000).astype(np.float64)
    z = z4.ravel()
    n = z.size
    assert abs(z.mean()) < 4 / math.sqrt(n)
    assert abs(z.var() - 1.0) < 0.02
    assert abs(((z - z.mean()) ** 4).mean() / z.var() ** 2 - 3.0) < 0.1
    assert sst.kstest(z, "norm").pvalue > 1e-3
    # every lane separately, and lanes pairwise uncorrelated
    for m in range(4):
        assert sst.kstest(z4[:, m], "norm").pvalue > 1e-3
    c = np.corrcoef(z4.T)
    assert np.abs(c - np.eye(4)).max() < 0.03


def test_gaussian_pairs_are_box_muller_of_their_own_words(oracle):
    """radius^2 of lanes (0,1) is -2 ln u(word 0), their angle is 2 pi u(word 1);
    lanes (2,3) use words 2 and 3.  Pins which word feeds which lane and which
    lane carries the cosine."""
    rng = np.random.default_rng(5)
    for _ in range(200):
        words = [int(w) for w in rng.integers(0, 2**32, 4)]
        z = oracle.noise4(words, 0).astype(np.float64)
        for pair in range(2):
            ua = float(brute.u01_fraction(words[2 * pair]))
            ub = float(brute.u01_fraction(words[2 * pair + 1]))
            r2 = z[2 * pair] ** 2 + z[2 * pair + 1] ** 2
            assert r2 == pytest.approx(-2.0 * math.log(ua), rel=1e-5, abs=1e-9)
            ang = math.atan2(z[2 * pair + 1], z[2 * pair]) % (2 * math.pi)
            diff = abs(ang - 2 * math.pi * ub)
            assert min(diff, 2 * math.pi - diff) < 1e-4 + 1e-6 / max(math.sqrt(r2), 1e-3)


def test_fill_distributions_and_slicing(oracle):
    seed = 0x161104581
    n = 40000
    h = oracle.fill(n, seed, oracle.STREAM_H)
    assert h.min() >= 0.1 and h.max() <= 1.0
    assert abs(h.mean() - 0.55) < 0.01
    assert abs(h.var() - 0.9 ** 2 / 12) < 0.003
    # h = fma(0.9, u, 0.1) exactly, with u from word (j % 4) of the block for quad j // 4
    for j in (0, 1, 2, 3, 4, 777, 39999):
        w = brute.philox4((j // 4, 0, 0, oracle.STREAM_H), (seed & 0xFFFFFFFF, seed >> 32))[j % 4]
        want = brute.f32_fma(Fraction(float(np.float32(0.9))), brute.u01_fraction(w), Fraction(float(np.float32(0.1))))
        assert Fraction(float(h[j])) == want
    for which in (oracle.STREAM_XSTAR, oracle.STREAM_X0):
        z = oracle.fill(n, seed, which).astype(np.float64)
        assert sst.kstest(z, "norm").pvalue > 1e-3
    a = oracle.fill(n, seed, oracle.STREAM_XSTAR)
    b = oracle.fill(n, seed, oracle.STREAM_X0)
    assert abs(np.corrcoef(a, b)[0, 1]) < 0.03          # different streams
    assert not np.array_equal(a, oracle.fill(n, seed + 1, oracle.STREAM_XSTAR))
    # a slice starting at an unaligned global column equals that part of the whole
    for col0, m in ((0, 17), (5, 1000), (1023, 514), (39990, 10)):
        for which in (oracle.STREAM_XSTAR, oracle.STREAM_H, oracle.STREAM_X0):
            whole = oracle.fill(n, seed, which)
            assert np.array_equal(oracle.fill(m, seed, which, col0=col0), whole[col0:col0 + m])
    with pytest.raises(ValueError):
        oracle.fill(4, seed, 0)


def test_perm_is_valid_and_matches_bigint_restatement(oracle):
    seed = 0x161104581
    for k in list(range(1, 40)) + [64, 100, 128, 257, 512]:
        for step in (0, 1, 12345):
            p = oracle.make_perm(seed, step, k)
            assert brute.is_permutation([int(t) for t in p])
            assert [int(t) for t in p] == brute.make_perm(seed, step, k)
    assert not np.array_equal(oracle.make_perm(seed, 0, 32), oracle.make_perm(seed, 1, 32))
    assert not np.array_equal(oracle.make_perm(seed, 0, 32), oracle.make_perm(seed + 1, 0, 32))
    with pytest.raises(ValueError):
        oracle.make_perm(seed, 0, 0)


@pytest.mark.parametrize("k", [3, 4])
def test_perm_is_uniform_over_all_outcomes(oracle, k):
    n = 24000
    counts = {}
    fixed = 0
    for step in range(n):
        p = tuple(int(t) for t in oracle.make_perm(99, step, k))
        counts[p] = counts.get(p, 0) + 1
        fixed += sum(1 for i, t in enumerate(p) if i == t)
    nperm = math.factorial(k)
    assert len(counts) == nperm
    obs = np.array(list(counts.values()), dtype=np.float64)
    chi2 = ((obs - n / nperm) ** 2 / (n / nperm)).sum()
    assert sst.chi2.sf(chi2, nperm - 1) > 1e-4
    assert abs(fixed / n - 1.0) < 0.05      # a uniform permutation has one fixed point on average
