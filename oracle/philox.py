"""Philox4x32-10 and the samplers built on it (oracle side).

Philox4x32-10 is the counter-based generator of Salmon, Moraes, Dror and Shaw
("Parallel random numbers: as easy as 1, 2, 3", SC'11), restated here from
its published description: ten rounds; one round maps (c0,c1,c2,c3) under
key (k0,k1) to (hi(M1*c2)^c1^k0, lo(M1*c2), hi(M0*c0)^c3^k1, lo(M0*c0));
the key is advanced by the Weyl constants (W0, W1) between rounds.

Keying used by the scheme (the paper is silent on randomness; this is the
reading stated in the design notes):
    key     = (seed & 0xffffffff, seed >> 32)
    counter = (block, ciphertext index, client id, tag)
tags: 0x00 secret s, 0x01 public-key error e, 0x10+j uniform a_j,
      0x20 ephemeral u, 0x21 e0, 0x22 e1.
Key generation uses ciphertext index = client id = 0.

Samplers are position-addressable (no rejection loops):
  ternary : coefficient k <- word (k mod 4) of block k//4; t = (x*3)>>32; value t-1
  CBD(eta): coefficient k <- block k//2, words (2(k&1), 2(k&1)+1);
            value popcount(w_a & (2^eta-1)) - popcount(w_b & (2^eta-1))
  uniform : coefficient k <- block k//2, x = w_hi*2^32 + w_lo with
            (w_lo, w_hi) = words (2(k&1), 2(k&1)+1); value x mod q
"""
from __future__ import annotations

import numpy as np

M0 = np.uint64(0xD2511F53)
M1 = np.uint64(0xCD9E8D57)
W0 = 0x9E3779B9
W1 = 0xBB67AE85
_MASK = np.uint64(0xFFFFFFFF)
_S32 = np.uint64(32)

TAG_S, TAG_EPK, TAG_A0, TAG_U, TAG_E0, TAG_E1 = 0x00, 0x01, 0x10, 0x20, 0x21, 0x22


def philox4x32_10(counters, key):
    """counters: (..., 4) integers < 2^32; key: (k0, k1). Returns (..., 4) uint32."""
    c = np.asarray(counters, dtype=np.uint64)
    c0, c1, c2, c3 = (c[..., i].copy() for i in range(4))
    k0, k1 = int(key[0]) & 0xFFFFFFFF, int(key[1]) & 0xFFFFFFFF
    for _ in range(10):
        p0 = M0 * c0
        p1 = M1 * c2
        hi0, lo0 = p0 >> _S32, p0 & _MASK
        hi1, lo1 = p1 >> _S32, p1 & _MASK
        c0, c1, c2, c3 = hi1 ^ c1 ^ np.uint64(k0), lo1, hi0 ^ c3 ^ np.uint64(k1), lo0
        k0 = (k0 + W0) & 0xFFFFFFFF
        k1 = (k1 + W1) & 0xFFFFFFFF
    return np.stack([c0, c1, c2, c3], axis=-1).astype(np.uint32)


def _blocks(seed: int, n_blocks: int, ct_index: int, client_id: int, tag: int):
    ctr = np.zeros((n_blocks, 4), dtype=np.uint64)
    ctr[:, 0] = np.arange(n_blocks, dtype=np.uint64)
    ctr[:, 1] = ct_index
    ctr[:, 2] = client_id
    ctr[:, 3] = tag
    key = (seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    return philox4x32_10(ctr, key)


def _popcount32(x):
    x = x.astype(np.uint64)
    cnt = np.zeros(x.shape, dtype=np.int64)
    for b in range(32):
        cnt += ((x >> np.uint64(b)) & np.uint64(1)).astype(np.int64)
    return cnt


def sample_ternary(seed, n_coeff, ct_index, client_id, tag):
    """n_coeff values in {-1,0,1} (int64)."""
    words = _blocks(seed, (n_coeff + 3) // 4, ct_index, client_id, tag).reshape(-1)[:n_coeff]
    t = (words.astype(np.uint64) * np.uint64(3)) >> _S32
    return t.astype(np.int64) - 1


def sample_cbd(seed, n_coeff, eta, ct_index, client_id, tag):
    """n_coeff centred-binomial values in [-eta, eta] (int64); eta = 0 gives zeros."""
    if eta == 0:
        return np.zeros(n_coeff, dtype=np.int64)
    assert 0 < eta <= 32
    w = _blocks(seed, (n_coeff + 1) // 2, ct_index, client_id, tag).reshape(-1, 2)[:n_coeff]
    mask = np.uint32((1 << eta) - 1)
    return _popcount32(w[:, 0] & mask) - _popcount32(w[:, 1] & mask)


def sample_uniform(seed, n_coeff, q, ct_index, client_id, tag):
    """n_coeff values in [0, q) (int64), q < 2^31."""
    w = _blocks(seed, (n_coeff + 1) // 2, ct_index, client_id, tag).reshape(-1, 2)[:n_coeff]
    x = (w[:, 1].astype(np.uint64) << _S32) | w[:, 0].astype(np.uint64)
    return (x % np.uint64(q)).astype(np.int64)
