"""CKKS slot encoding / decoding for real vectors (oracle side).

The paper packs a fixed number of parameters per ciphertext (its "packing
batch size", Section "Default Crypto Parameters") and relies on CKKS handling
approximate numbers (Section "Homomorphic Encryption"); it does not spell out
the encoding.  The textbook map is used: slot j of a plaintext polynomial m
is m evaluated at zeta^(g_j), zeta = exp(i*pi/N), g_j = 5^j mod 2N, and the
other half of the odd powers carries the complex conjugates.  For a real
slot vector z in R^n (n = N/2) and scale Delta that gives

    encode:  m_k = rint( (2*Delta/N) * sum_j z_j cos(pi * g_j * k / N) ),  0 <= k < N
    decode:  z_j = (1/Delta) * sum_k v_k cos(pi * g_j * k / N)

(the imaginary part of the evaluation is the conjugate slot's business and is
dropped).  rint is round-half-to-even on the float64 value.

`encode_def` / `decode_def` are these sums written out with one float64
matrix product; `encode_fft` / `decode_fft` reach the same values through
numpy's FFT and are pinned to the definitions by the tests.
"""
from __future__ import annotations

from functools import lru_cache

import numpy as np


@lru_cache(maxsize=None)
def rotation_group(log2_n: int):
    """g_j = 5^j mod 2N for j < N/2 (int64)."""
    n_ring = 1 << log2_n
    g = np.empty(n_ring // 2, dtype=np.int64)
    x = 1
    for j in range(n_ring // 2):
        g[j] = x
        x = x * 5 % (2 * n_ring)
    return g


@lru_cache(maxsize=4)
def _cos_matrix(log2_n: int):
    """C[k, j] = cos(pi * g_j * k / N); the angle is reduced exactly mod 2N first."""
    n_ring = 1 << log2_n
    g = rotation_group(log2_n)
    k = np.arange(n_ring, dtype=np.int64).reshape(-1, 1)
    r = (k * g.reshape(1, -1)) % (2 * n_ring)
    return np.cos(np.pi * r.astype(np.float64) / n_ring)


def encode_def(z, log2_n: int, scale_bits: int):
    """Definition of the encoder: direct O(N*n) cosine sum, float64, then rint."""
    n_ring = 1 << log2_n
    z = np.asarray(z, dtype=np.float64)
    assert z.shape == (n_ring // 2,)
    val = (2.0 * float(1 << scale_bits) / n_ring) * (_cos_matrix(log2_n) @ z)
    return np.rint(val).astype(np.int64)


def decode_def(v, log2_n: int, scale_bits: int):
    """Definition of the decoder: direct cosine sum over the N coefficients."""
    v = np.asarray(v, dtype=np.float64)
    return (_cos_matrix(log2_n).T @ v) / float(1 << scale_bits)


def _bins(log2_n: int):
    """FFT bin of slot j.  With c_k = m_k + i*m_{k+n} (X^n evaluates to i at every
    zeta^(g_j) because g_j = 1 mod 4) the slot value is
    sum_k c_k zeta^k exp(2*pi*i*t_j*k/n), t_j = (g_j - 1)/4."""
    return (rotation_group(log2_n) - 1) // 4


def encode_fft(z, log2_n: int, scale_bits: int):
    n_ring = 1 << log2_n
    n = n_ring // 2
    z = np.asarray(z, dtype=np.float64)
    y = np.zeros(n, dtype=np.complex128)
    y[_bins(log2_n)] = z
    c = np.fft.fft(y) / n                                     # sum_t y_t exp(-2 pi i t k / n) / n
    c = c * np.exp(-1j * np.pi * np.arange(n) / n_ring)       # times zeta^-k
    c = c * float(1 << scale_bits)
    return np.rint(np.concatenate([c.real, c.imag])).astype(np.int64)


def decode_fft(v, log2_n: int, scale_bits: int):
    n_ring = 1 << log2_n
    n = n_ring // 2
    v = np.asarray(v, dtype=np.float64)
    c = (v[:n] + 1j * v[n:]) * np.exp(1j * np.pi * np.arange(n) / n_ring)
    full = np.fft.ifft(c) * n                                 # sum_k c_k exp(+2 pi i t k / n)
    return full[_bins(log2_n)].real / float(1 << scale_bits)
