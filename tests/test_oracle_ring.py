"""Pins for the oracle's ring arithmetic: brute force, definitions, invariants."""
import numpy as np
import pytest

from oracle import ring
from oracle.params import Params


def _adversarial(n_ring, q, rs):
    yield rs.integers(0, q, n_ring)
    yield np.full(n_ring, q - 1, dtype=np.int64)
    v = np.zeros(n_ring, dtype=np.int64)
    v[-1] = q - 1
    yield v
    yield np.arange(n_ring, dtype=np.int64) % q


@pytest.mark.parametrize("log2_n", [3, 4, 6, 8])
def test_transform_equals_evaluation_and_product_equals_schoolbook(log2_n):
    n_ring = 1 << log2_n
    p = Params(log2_n, 3)
    rs = np.random.default_rng(log2_n)
    for j, q in enumerate(p.primes):
        psi = p.psi(j)
        for a in _adversarial(n_ring, q, rs):
            fa = ring.ntt(a, q, psi)
            if log2_n <= 6:
                assert np.array_equal(fa, ring.ntt_def(a, q, psi))
            assert np.array_equal(ring.intt(fa, q, psi), a)
            for b in _adversarial(n_ring, q, rs):
                ref = ring.negacyclic_mul_schoolbook(a, b, q) if log2_n <= 6 else ring.negacyclic_mul_def(a, b, q)
                assert np.array_equal(ring.negacyclic_mul(a, b, q, psi), ref)
                if log2_n <= 4:
                    assert np.array_equal(ring.negacyclic_mul_def(a, b, q), ref)


@pytest.mark.parametrize("log2_n,limbs", [(13, 3), (14, 4)])
def test_full_size_rings(log2_n, limbs):
    n_ring = 1 << log2_n
    p = Params(log2_n, limbs)
    rs = np.random.default_rng(99)
    for j, q in enumerate(p.primes):
        psi = p.psi(j)
        a = rs.integers(0, q, n_ring)
        assert np.array_equal(ring.intt(ring.ntt(a, q, psi), q, psi), a)
        assert np.array_equal(ring.ntt(ring.intt(a, q, psi), q, psi), a)
        # X * a(X): negacyclic shift with the wrapped coefficient negated
        x = np.zeros(n_ring, dtype=np.int64)
        x[1] = 1
        shifted = np.concatenate([[(q - a[-1]) % q], a[:-1]])
        assert np.array_equal(ring.negacyclic_mul(a, x, q, psi), shifted)
        # linearity of the transform
        b = rs.integers(0, q, n_ring)
        assert np.array_equal(ring.ntt((a + 3 * b) % q, q, psi),
                              (ring.ntt(a, q, psi) + 3 * ring.ntt(b, q, psi)) % q)
    # convolution theorem against the linear-convolution definition, one limb, dense operands
    q, psi = p.primes[-1], p.psi(limbs - 1)
    a, b = rs.integers(0, q, n_ring), rs.integers(0, q, n_ring)
    assert np.array_equal(ring.negacyclic_mul(a, b, q, psi), ring.negacyclic_mul_def(a, b, q))


def test_transform_output_order():
    """Entry i is the evaluation at psi^(2*brev(i)+1): check on the monomial X."""
    p = Params(4, 3)
    q, psi = p.primes[0], p.psi(0)
    x = np.zeros(16, dtype=np.int64)
    x[1] = 1
    out = ring.ntt(x, q, psi)
    assert [int(v) for v in out] == [pow(psi, 2 * ring.bit_reverse(i, 4) + 1, q) for i in range(16)]
