"""Ring and modulus-chain parameters (oracle side).

The paper names only the scheme (CKKS) and four defaults (multiplicative
depth 1, a scaling-factor bit width, a packing batch size, 128-bit security;
Section "Default Crypto Parameters").  The ring-level choices used here:
  * R = Z[X]/(X^N + 1), N a power of two, n = N/2 slots per ciphertext
    (the "packing batch size");
  * an RNS chain q_0 > q_1 > ... > q_{L-1} of the largest primes below 2^31
    with q = 1 (mod 2N);
  * psi_j = the smallest primitive 2N-th root of unity modulo q_j.
Everything is re-derived here from these definitions by search; nothing is
copied from a table.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from functools import lru_cache

_MR_BASES = (2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37)  # deterministic below 3.3e24


def is_prime(n: int) -> bool:
    """Deterministic Miller-Rabin for n < 3.3e24."""
    if n < 2:
        return False
    for p in _MR_BASES:
        if n % p == 0:
            return n == p
    d, r = n - 1, 0
    while d % 2 == 0:
        d //= 2
        r += 1
    for a in _MR_BASES:
        x = pow(a, d, n)
        if x in (1, n - 1):
            continue
        for _ in range(r - 1):
            x = x * x % n
            if x == n - 1:
                break
        else:
            return False
    return True


@lru_cache(maxsize=None)
def find_primes(log2_n: int, count: int, below: int = 1 << 31) -> tuple:
    """The `count` largest primes q < `below` with q = 1 (mod 2N), descending."""
    two_n = 2 << log2_n
    q = (below - 1) // two_n * two_n + 1
    if q >= below:
        q -= two_n
    out = []
    while len(out) < count:
        if q <= two_n:
            raise ValueError("not enough primes")
        if is_prime(q):
            out.append(q)
        q -= two_n
    return tuple(out)


@lru_cache(maxsize=None)
def smallest_primitive_2n_root(q: int, log2_n: int) -> int:
    """Smallest psi with psi^N = -1 (mod q) (its order is then exactly 2N).

    Any x with c = x^((q-1)/2N) satisfying c^N = -1 gives one primitive 2N-th
    root; the others are its odd powers, so the minimum over those N values is
    the smallest one.
    """
    n_ring = 1 << log2_n
    assert (q - 1) % (2 * n_ring) == 0
    for x in range(2, q):
        c = pow(x, (q - 1) // (2 * n_ring), q)
        if pow(c, n_ring, q) == q - 1:
            break
    else:
        raise ValueError("no root")
    best, cur, c2 = c, c, c * c % q
    for _ in range(n_ring - 1):
        cur = cur * c2 % q
        best = min(best, cur)
    return best


@dataclass(frozen=True)
class Params:
    """Public crypto context: ring degree, chain, scale, noise parameter."""
    log2_n: int
    n_limbs: int
    scale_bits: int = 30
    cbd_eta: int = 21
    primes: tuple = field(default=())

    def __post_init__(self):
        if not self.primes:
            object.__setattr__(self, "primes", find_primes(self.log2_n, self.n_limbs))
        assert len(self.primes) == self.n_limbs
        for q in self.primes:
            assert is_prime(q) and q < (1 << 31) and (q - 1) % (2 * self.N) == 0

    @property
    def N(self) -> int:
        return 1 << self.log2_n

    @property
    def n_slots(self) -> int:
        return self.N // 2

    @property
    def delta(self) -> int:
        return 1 << self.scale_bits

    def psi(self, j: int) -> int:
        return smallest_primitive_2n_root(self.primes[j], self.log2_n)
