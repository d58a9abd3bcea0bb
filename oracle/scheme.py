"""RNS-CKKS key generation, encryption, weighted aggregation, rescale, decryption.

Follows Algorithm 1 of the paper for what is computed:
    key authority : (pk, sk) <- HE.KeyGen
    client        : [W_i] <- HE.Enc(pk, M . W_i) + (1-M) . W_i
    server        : [W_glob] <- sum_i alpha_i [[M . W_i]] + sum_i alpha_i (1-M) . W_i
    client        : W <- HE.Dec(sk, M . [W_glob]) + (1-M) . [W_glob]
with plaintext aggregation weights and one multiplicative depth (Section
"Algorithm for HE-Based Federated Aggregation").  The ring-level form of each
HE call is the textbook RLWE one, since the paper does not print it:

  KeyGen : s ternary; a_j uniform in R_{q_j}; e <- CBD(eta);
           b_j = -(a_j * s) + e (mod q_j);  pk = (b, a), sk = s.
  Enc    : u ternary, e0, e1 <- CBD(eta);
           c0_j = b_j * u + e0 + m,  c1_j = a_j * u + e1  (mod q_j).
  Eval   : w_i = rint(alpha_i * q_{L-1}) (float64 product, round-half-even);
           acc_{p,j} = sum_i w_i * ct_i[p][j]  (mod q_j) for all L limbs; then
           rescale drops q_{L-1}: with r~ the centred residue of acc_{p,L-1},
           out_{p,j} = (acc_{p,j} - r~) * q_{L-1}^{-1} (mod q_j), j < L-1.
  Dec    : d_j = c0_j + c1_j * s (mod q_j), j < L-1;  v = centred CRT lift in
           (-Q'/2, Q'/2], Q' = prod_{j<L-1} q_j.

Ciphertexts are kept in the coefficient domain with residues in [0, q_j),
layout [poly][limb][N]; `*` is the negacyclic product.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

from . import philox as rng
from .params import Params
from .ring import negacyclic_mul


@dataclass
class KeyPair:
    s: np.ndarray          # (N,) int64 in {-1,0,1}
    pk_b: np.ndarray       # (L, N) int64 residues
    pk_a: np.ndarray       # (L, N) int64 residues
    e: np.ndarray          # (N,) int64, kept for the tests' invariants


def keygen(p: Params, seed: int) -> KeyPair:
    n_ring = p.N
    s = rng.sample_ternary(seed, n_ring, 0, 0, rng.TAG_S)
    e = rng.sample_cbd(seed, n_ring, p.cbd_eta, 0, 0, rng.TAG_EPK)
    pk_a = np.zeros((p.n_limbs, n_ring), dtype=np.int64)
    pk_b = np.zeros((p.n_limbs, n_ring), dtype=np.int64)
    for j, q in enumerate(p.primes):
        a = rng.sample_uniform(seed, n_ring, q, 0, 0, rng.TAG_A0 + j)
        a_s = negacyclic_mul(a, s % q, q, p.psi(j))
        pk_a[j] = a
        pk_b[j] = (e - a_s) % q
    return KeyPair(s=s, pk_b=pk_b, pk_a=pk_a, e=e)


def encrypt(p: Params, keys: KeyPair, m, seed: int, client_id: int, ct_index: int):
    """m: (N,) signed integers (the encoded plaintext).  Returns (2, L, N) int64."""
    n_ring = p.N
    m = np.asarray(m, dtype=np.int64)
    u = rng.sample_ternary(seed, n_ring, ct_index, client_id, rng.TAG_U)
    e0 = rng.sample_cbd(seed, n_ring, p.cbd_eta, ct_index, client_id, rng.TAG_E0)
    e1 = rng.sample_cbd(seed, n_ring, p.cbd_eta, ct_index, client_id, rng.TAG_E1)
    ct = np.zeros((2, p.n_limbs, n_ring), dtype=np.int64)
    for j, q in enumerate(p.primes):
        uq = u % q
        ct[0, j] = (negacyclic_mul(keys.pk_b[j], uq, q, p.psi(j)) + e0 + m) % q
        ct[1, j] = (negacyclic_mul(keys.pk_a[j], uq, q, p.psi(j)) + e1) % q
    return ct


def integer_weights(p: Params, alpha):
    """w_i = rint(alpha_i * q_{L-1}), float64 product, ties to even."""
    alpha = np.asarray(alpha, dtype=np.float64)
    w = np.rint(alpha * np.float64(p.primes[-1]))
    return [int(x) for x in w]


def weighted_sum(p: Params, cts, alpha):
    """acc[p][j] = sum_i w_i * ct_i[p][j] mod q_j, all L limbs.  cts: list of (2, L, N)."""
    w = integer_weights(p, alpha)
    acc = np.zeros_like(np.asarray(cts[0], dtype=np.int64))
    for j, q in enumerate(p.primes):
        for wi, ct in zip(w, cts):
            acc[:, j] = (acc[:, j] + (wi % q) * np.asarray(ct, dtype=np.int64)[:, j]) % q
    return acc


def rescale(p: Params, acc):
    """Drop the last limb with round-to-nearest.  (2, L, N) -> (2, L-1, N)."""
    q_last = p.primes[-1]
    r = np.asarray(acc, dtype=np.int64)[:, -1]
    r_c = np.where(r > (q_last - 1) // 2, r - q_last, r)
    out = np.zeros((2, p.n_limbs - 1, p.N), dtype=np.int64)
    for j, q in enumerate(p.primes[:-1]):
        inv = pow(q_last, q - 2, q)
        out[:, j] = ((acc[:, j] - r_c) % q) * inv % q
    return out


def aggregate(p: Params, cts, alpha):
    """Server-side weighted homomorphic FedAvg of K ciphertexts (same index)."""
    return rescale(p, weighted_sum(p, cts, alpha))


def sum_ciphertexts(p: Params, cts):
    """Weighing-on-the-client variant (Section "Comparison with Other FL Frameworks": learners scale
    their parameters locally, the server only adds): out[p][j] = sum_i ct_i[p][j] mod q_j, level kept."""
    acc = np.zeros_like(np.asarray(cts[0], dtype=np.int64))
    for j, q in enumerate(p.primes):
        for ct in cts:
            acc[:, j] = (acc[:, j] + np.asarray(ct, dtype=np.int64)[:, j]) % q
    return acc


def crt_centered(residues, primes):
    """Exact centred lift of (len(primes), N) residues to Python ints in (-Q/2, Q/2]."""
    big_q = 1
    for q in primes:
        big_q *= q
    n_ring = residues.shape[1]
    out = [0] * n_ring
    for j, q in enumerate(primes):
        qhat = big_q // q
        c = qhat * pow(qhat % q, q - 2, q)
        row = residues[j]
        for k in range(n_ring):
            out[k] += int(row[k]) * c
    half = big_q // 2   # Q odd: (-Q/2, Q/2] means v <= (Q-1)/2
    res = []
    for v in out:
        v %= big_q
        res.append(v - big_q if v > half else v)
    return res


def decrypt_residues(p: Params, keys: KeyPair, ct, level: int):
    """Dec before the lift: d_j = c0_j + c1_j * s mod q_j as (level, N) int64.  ct: (2, level, N)."""
    d = np.zeros((level, p.N), dtype=np.int64)
    for j in range(level):
        q = p.primes[j]
        d[j] = (ct[0, j] + negacyclic_mul(ct[1, j], keys.s % q, q, p.psi(j))) % q
    return d


def decrypt(p: Params, keys: KeyPair, ct, level: int):
    """ct: (2, level, N).  Returns the centred integer plaintext as a list of Python ints."""
    return crt_centered(decrypt_residues(p, keys, ct, level), p.primes[:level])
