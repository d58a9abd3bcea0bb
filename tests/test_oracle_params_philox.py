"""Pins for the oracle's parameter search, Philox4x32-10 and the samplers."""
import os

import numpy as np
import pytest

from oracle import params as op
from oracle import philox as rng

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def _trial_prime(n):
    if n < 2:
        return False
    i = 2
    while i * i <= n:
        if n % i == 0:
            return False
        i += 1
    return True


@pytest.mark.parametrize("log2_n,count", [(13, 3), (14, 4), (3, 3), (4, 3)])
def test_primes_are_the_largest(log2_n, count):
    two_n = 2 << log2_n
    primes = op.find_primes(log2_n, count)
    assert list(primes) == sorted(primes, reverse=True)
    # independent check by trial division of every candidate down to the last prime
    expect = []
    q = ((1 << 31) - 1) // two_n * two_n + 1
    while len(expect) < count:
        if q < (1 << 31) and _trial_prime(q):
            expect.append(q)
        q -= two_n
    assert list(primes) == expect
    assert all(p < (1 << 31) and p % two_n == 1 for p in primes)


def test_miller_rabin_on_known_values():
    assert op.is_prime(2147483647) and op.is_prime(998244353) and op.is_prime(2)
    assert not op.is_prime(2147483649) and not op.is_prime(1)
    assert not op.is_prime(3215031751)          # strong pseudoprime to bases 2,3,5,7
    assert not op.is_prime(561) and not op.is_prime(2147352577 * 3)


@pytest.mark.parametrize("log2_n,count", [(13, 3), (14, 4), (4, 3)])
def test_roots(log2_n, count):
    n_ring = 1 << log2_n
    p = op.Params(log2_n, count)
    for j, q in enumerate(p.primes):
        psi = p.psi(j)
        assert pow(psi, n_ring, q) == q - 1 and pow(psi, 2 * n_ring, q) == 1
        if psi < 400000:   # smallest: nothing below it qualifies (direct scan)
            assert all(pow(x, n_ring, q) != q - 1 for x in range(2, psi))
        # all 2N-th roots of -1 are psi^odd: none of them is smaller
        assert all(pow(psi, k, q) >= psi for k in range(1, 2 * n_ring, max(2, 2 * (n_ring // 512))))


def test_philox_known_answers():
    rows = [ln.split() for ln in open(GOLDEN) if ln.strip() and not ln.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        vals = [int(x, 16) for x in r]
        out = rng.philox4x32_10(np.array(vals[0:4]), (vals[4], vals[5]))
        assert [int(x) for x in out] == vals[6:10]


def test_philox_scalar_reimplementation():
    """A second, scalar, Python-int implementation written from the round description."""
    def scalar(c, k):
        c = list(c)
        k = list(k)
        for _ in range(10):
            p0 = 0xD2511F53 * c[0]
            p1 = 0xCD9E8D57 * c[2]
            c = [(p1 >> 32) ^ c[1] ^ k[0], p1 & 0xFFFFFFFF, (p0 >> 32) ^ c[3] ^ k[1], p0 & 0xFFFFFFFF]
            k = [(k[0] + 0x9E3779B9) & 0xFFFFFFFF, (k[1] + 0xBB67AE85) & 0xFFFFFFFF]
        return c
    rs = np.random.default_rng(5)
    ctr = rs.integers(0, 1 << 32, size=(200, 4), dtype=np.uint64)
    key = (0x12345678, 0x9ABCDEF0)
    out = rng.philox4x32_10(ctr, key)
    for i in range(200):
        assert [int(x) for x in out[i]] == scalar([int(x) for x in ctr[i]], key)


def test_word_uniformity_and_sampler_statistics():
    n = 1 << 20
    words = rng._blocks(12345, n // 4, 3, 2, rng.TAG_U).reshape(-1)
    hist = np.bincount(words >> 24, minlength=256)          # chi-square on the top byte
    chi2 = float(((hist - n / 256) ** 2 / (n / 256)).sum())
    assert chi2 < 255 + 6 * np.sqrt(2 * 255)
    t = rng.sample_ternary(12345, n, 3, 2, rng.TAG_U)
    freq = np.bincount(t + 1, minlength=3) / n
    assert set(np.unique(t)) == {-1, 0, 1} and np.abs(freq - 1 / 3).max() < 3e-3
    e = rng.sample_cbd(12345, n, 21, 3, 2, rng.TAG_E0)
    assert e.min() >= -21 and e.max() <= 21
    assert abs(e.mean()) < 0.02 and abs(e.var() - 10.5) < 0.105
    assert np.all(rng.sample_cbd(1, 64, 0, 0, 0, rng.TAG_E0) == 0)
    q = 2147352577
    a = rng.sample_uniform(12345, n, q, 0, 0, rng.TAG_A0)
    assert a.min() >= 0 and a.max() < q and abs(a.mean() / q - 0.5) < 2e-3


def test_samplers_follow_their_word_layout():
    """Each coefficient is a fixed function of one Philox block: check against hand-picked words."""
    seed, ct, cl = (7 << 32) | 9, 11, 5
    blk = lambda b, tag: [int(x) for x in rng.philox4x32_10(np.array([b, ct, cl, tag]), (9, 7))]
    t = rng.sample_ternary(seed, 10, ct, cl, rng.TAG_U)
    for k in range(10):
        assert t[k] == ((blk(k // 4, rng.TAG_U)[k % 4] * 3) >> 32) - 1
    e = rng.sample_cbd(seed, 9, 21, ct, cl, rng.TAG_E1)
    for k in range(9):
        w = blk(k // 2, rng.TAG_E1)
        wa, wb = w[2 * (k & 1)], w[2 * (k & 1) + 1]
        assert e[k] == bin(wa & 0x1FFFFF).count("1") - bin(wb & 0x1FFFFF).count("1")
    q = 2146041857
    a = rng.sample_uniform(seed, 9, q, 0, 0, rng.TAG_A0 + 3)
    for k in range(9):
        w = [int(x) for x in rng.philox4x32_10(np.array([k // 2, 0, 0, rng.TAG_A0 + 3]), (9, 7))]
        assert a[k] == ((w[2 * (k & 1) + 1] << 32) | w[2 * (k & 1)]) % q
    # streams with different tags / clients / ciphertext indices differ
    base = rng.sample_ternary(seed, 256, ct, cl, rng.TAG_U)
    assert not np.array_equal(base, rng.sample_ternary(seed, 256, ct + 1, cl, rng.TAG_U))
    assert not np.array_equal(base, rng.sample_ternary(seed, 256, ct, cl + 1, rng.TAG_U))
    assert not np.array_equal(base, rng.sample_ternary(seed, 256, ct, cl, rng.TAG_S))
    assert not np.array_equal(base, rng.sample_ternary(seed + (1 << 32), 256, ct, cl, rng.TAG_U))
