"""Arithmetic in R_q = Z_q[X]/(X^N + 1) (oracle side).

Two layers:
  * definitions -- the negacyclic product as a linear convolution folded with
    X^N = -1, and the number-theoretic transform as plain evaluation of the
    polynomial at the odd powers of psi;
  * a fast iterative NTT/INTT (numpy uint64), which the tests pin to the
    definitions by brute force on small rings and through the convolution
    theorem on the full-size rings.

Output order of the transform (fixed so that two implementations can be
compared value by value): entry i holds a(psi^(2*brev(i)+1)), where brev is
the log2(N)-bit reversal and psi the smallest primitive 2N-th root.
"""
from __future__ import annotations

import numpy as np


def bit_reverse(i: int, bits: int) -> int:
    r = 0
    for _ in range(bits):
        r = (r << 1) | (i & 1)
        i >>= 1
    return r


def negacyclic_mul_def(a, b, q: int):
    """Definition: c = a*b mod (X^N + 1, q), via the full linear convolution.

    a, b: integer arrays with entries in [0, q), q < 2^31.  The convolution is
    taken exactly in int64 by splitting b into 11-bit digits, so that no partial
    sum exceeds N * 2^31 * 2^11 < 2^63 for N <= 2^16.
    """
    a = np.asarray(a, dtype=np.int64)
    b = np.asarray(b, dtype=np.int64)
    n_ring = a.shape[0]
    assert b.shape[0] == n_ring and n_ring <= (1 << 16)
    total = np.zeros(n_ring, dtype=object)
    for d in range(3):
        digit = (b >> (11 * d)) & 0x7FF
        full = np.convolve(a, digit)                      # length 2N-1, exact
        full = np.concatenate([full, np.zeros(1, dtype=np.int64)])
        folded = (full[:n_ring] % q) - (full[n_ring:] % q)  # X^N = -1
        total = total + folded.astype(object) * (1 << (11 * d))
    return np.array([int(x) % q for x in total], dtype=np.int64)


def negacyclic_mul_schoolbook(a, b, q: int):
    """Pure-Python O(N^2) double loop; for tiny rings only."""
    n_ring = len(a)
    c = [0] * n_ring
    for i in range(n_ring):
        for j in range(n_ring):
            k = i + j
            term = int(a[i]) * int(b[j])
            if k >= n_ring:
                c[k - n_ring] -= term
            else:
                c[k] += term
    return np.array([x % q for x in c], dtype=np.int64)


def ntt_def(a, q: int, psi: int):
    """Definition: out[i] = a(psi^(2*brev(i)+1)) mod q, by Horner; small N only."""
    n_ring = len(a)
    bits = n_ring.bit_length() - 1
    out = np.zeros(n_ring, dtype=np.int64)
    for i in range(n_ring):
        x = pow(psi, 2 * bit_reverse(i, bits) + 1, q)
        acc = 0
        for coeff in reversed([int(v) for v in a]):
            acc = (acc * x + coeff) % q
        out[i] = acc
    return out


def _psi_rev_table(n_ring: int, q: int, root: int):
    bits = n_ring.bit_length() - 1
    pw = [1] * n_ring
    for k in range(1, n_ring):
        pw[k] = pw[k - 1] * root % q
    return np.array([pw[bit_reverse(k, bits)] for k in range(n_ring)], dtype=np.uint64)


_TABLES = {}


def _tables(n_ring: int, q: int, psi: int):
    key = (n_ring, q, psi)
    if key not in _TABLES:
        _TABLES[key] = (_psi_rev_table(n_ring, q, psi),
                        _psi_rev_table(n_ring, q, pow(psi, q - 2, q)))
    return _TABLES[key]


def ntt(a, q: int, psi: int):
    """Fast forward negacyclic NTT (decimation in time with merged psi powers).

    Natural-order coefficients in, bit-reversed evaluations out (same order as
    ntt_def).  Stage with m blocks: block i is multiplied by psi^brev(m+i).
    """
    x = np.asarray(a, dtype=np.uint64).copy()
    n_ring = x.shape[0]
    fwd, _ = _tables(n_ring, q, psi)
    qq = np.uint64(q)
    m, t = 1, n_ring // 2
    while m < n_ring:
        v = x.reshape(m, 2, t)
        w = fwd[m:2 * m].reshape(m, 1)
        lo = v[:, 0, :]
        hi = (v[:, 1, :] * w) % qq
        v[:, 0, :], v[:, 1, :] = (lo + hi) % qq, (lo + qq - hi) % qq
        m, t = 2 * m, t // 2
    return x.astype(np.int64)


def intt(a_hat, q: int, psi: int):
    """Inverse of ntt(): bit-reversed evaluations in, natural coefficients out."""
    x = np.asarray(a_hat, dtype=np.uint64).copy()
    n_ring = x.shape[0]
    _, inv = _tables(n_ring, q, psi)
    qq = np.uint64(q)
    m, t = n_ring // 2, 1
    while m >= 1:
        v = x.reshape(m, 2, t)
        w = inv[m:2 * m].reshape(m, 1)
        lo, hi = v[:, 0, :].copy(), v[:, 1, :].copy()
        v[:, 0, :] = (lo + hi) % qq
        v[:, 1, :] = ((lo + qq - hi) % qq) * w % qq
        m, t = m // 2, 2 * t
    n_inv = np.uint64(pow(n_ring, q - 2, q))
    return ((x * n_inv) % qq).astype(np.int64)


def negacyclic_mul(a, b, q: int, psi: int):
    """Negacyclic product through the transform (pinned to negacyclic_mul_def)."""
    fa = ntt(np.asarray(a, dtype=np.int64) % q, q, psi).astype(np.uint64)
    fb = ntt(np.asarray(b, dtype=np.int64) % q, q, psi).astype(np.uint64)
    return intt((fa * fb) % np.uint64(q), q, psi)
