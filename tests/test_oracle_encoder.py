"""Pins for the oracle's CKKS encoder/decoder: closed forms and direct evaluation."""
import cmath

import numpy as np
import pytest

from oracle import encoder as enc


def _evaluate_slots(m, log2_n):
    """Independent formulation: evaluate the polynomial at zeta^(5^j) by complex Horner."""
    n_ring = 1 << log2_n
    out = []
    for j in range(n_ring // 2):
        x = cmath.exp(1j * cmath.pi * pow(5, j, 2 * n_ring) / n_ring)
        acc = 0j
        for c in reversed([float(v) for v in m]):
            acc = acc * x + c
        out.append(acc)
    return np.array(out)


SCALES = [30, 20, 12]


@pytest.mark.parametrize("scale_bits", SCALES)
@pytest.mark.parametrize("log2_n", [3, 4, 6])
def test_decode_is_evaluation_at_the_rotation_group(log2_n, scale_bits):
    rs = np.random.default_rng(log2_n)
    n_ring = 1 << log2_n
    m = rs.integers(-(1 << 28), 1 << 28, n_ring)
    ev = _evaluate_slots(m, log2_n) / (1 << scale_bits)
    for dec in (enc.decode_def, enc.decode_fft):
        assert np.allclose(dec(m, log2_n, scale_bits), ev.real, rtol=0, atol=1e-9 * 2.0 ** (30 - scale_bits))


@pytest.mark.parametrize("scale_bits", SCALES)
@pytest.mark.parametrize("log2_n", [3, 4, 6, 10, 11])
def test_encode_closed_forms(log2_n, scale_bits):
    n_ring = 1 << log2_n
    n = n_ring // 2
    for f in (enc.encode_def, enc.encode_fft):
        # constant vector -> constant polynomial
        m = f(np.full(n, 0.3125), log2_n, scale_bits)
        assert m[0] == int(0.3125 * (1 << scale_bits)) and np.all(m[1:] == 0)
        # unit vector e_j -> (2*Delta/N) cos(pi g_j k / N)
        for j in (0, 1, n - 1):
            z = np.zeros(n)
            z[j] = 1.0
            g = pow(5, j, 2 * n_ring)
            expect = [round((2.0 * (1 << scale_bits) / n_ring) * np.cos(np.pi * ((g * k) % (2 * n_ring)) / n_ring))
                      for k in range(n_ring)]
            assert np.abs(f(z, log2_n, scale_bits) - np.array(expect)).max() <= 1
        # linear up to rounding, odd in sign
        z = np.random.default_rng(1).normal(0, 0.05, n)
        assert np.array_equal(f(z, log2_n, scale_bits), -f(-z, log2_n, scale_bits))
        # the scale is a power of two: one more bit doubles the unrounded value, so the coefficients follow within rounding
        assert np.abs(f(z, log2_n, scale_bits) - 2 * f(z, log2_n, scale_bits - 1)).max() <= 2


@pytest.mark.parametrize("log2_n,scale_bits", [(3, 30), (4, 30), (8, 30), (13, 30), (14, 30), (4, 20), (11, 20), (13, 20), (11, 30)])
def test_fft_path_equals_definition_and_roundtrip(log2_n, scale_bits):
    n_ring = 1 << log2_n
    rs = np.random.default_rng(17 + log2_n)
    z = rs.normal(0, 0.05, n_ring // 2).astype(np.float32).astype(np.float64)
    m_def, m_fft = enc.encode_def(z, log2_n, scale_bits), enc.encode_fft(z, log2_n, scale_bits)
    assert np.abs(m_def - m_fft).max() <= 1 and (m_def != m_fft).mean() < 1e-3
    # a slot vector of variance s^2 gives coefficients of variance (2 Delta / N)^2 * n * s^2 / 2 = Delta^2 s^2 / N
    if n_ring >= 256:
        assert 0.8 < m_def.std() / ((1 << scale_bits) * 0.05 / np.sqrt(n_ring)) < 1.25
    # the slots of the rounded polynomial are the inputs up to the rounding error:
    # each coefficient is off by at most 1/2, a slot sums N of them against unit-modulus weights
    for dec in (enc.decode_def, enc.decode_fft):
        err = np.abs(dec(m_def, log2_n, scale_bits) - z)
        assert err.max() <= 0.5 * n_ring / (1 << scale_bits)
        assert err.max() <= 8 * np.sqrt(n_ring / 24.0) / (1 << scale_bits) + 1e-12
    # exact evaluation of the unrounded value for one coefficient with Python floats in higher care
    k = 5
    g = enc.rotation_group(log2_n)
    import math
    exact = math.fsum(float(z[j]) * math.cos(math.pi * ((int(g[j]) * k) % (2 * n_ring)) / n_ring)
                      for j in range(n_ring // 2)) * (2.0 * (1 << scale_bits) / n_ring)
    assert abs(m_def[k] - exact) <= 0.5 + 1e-6


def test_rotation_group_covers_residues_one_mod_four():
    for log2_n in (3, 4, 10, 14):
        g = enc.rotation_group(log2_n)
        n_ring = 1 << log2_n
        assert sorted(g.tolist()) == list(range(1, 2 * n_ring, 4))
