"""The oracle's pins must fail when a plausible mistake is planted in the oracle.

Each case replaces one oracle function (on the CPU, for the duration of the case) by a copy with
one planted mistake -- a dropped term, a wrong sign, a swapped operand, a wrong rounding, a wrong
index -- and runs the pin that is meant to catch it.  The pin has to raise.  (The unmodified pins
pass in their own test files; here only their power to reject is tested.)
"""
import numpy as np
import pytest

import test_oracle_encoder as pins_encoder
import test_oracle_fedavg as pins_fedavg
import test_oracle_params_philox as pins_philox
import test_oracle_ring as pins_ring
import test_oracle_scheme as pins_scheme
import test_oracle_select as pins_select
from oracle import encoder, fedavg, philox, ring, scheme, select
from oracle.params import Params


def _small_ctx():
    p = Params(6, 3)
    return p, scheme.keygen(p, 0xC0FFEE + 6)


# ---- planted mistakes -----------------------------------------------------------------------

def rescale_floor(p, acc):                      # rounds down instead of to nearest
    q_last = p.primes[-1]
    r = np.asarray(acc, dtype=np.int64)[:, -1]
    out = np.zeros((2, p.n_limbs - 1, p.N), dtype=np.int64)
    for j, q in enumerate(p.primes[:-1]):
        out[:, j] = ((acc[:, j] - r) % q) * pow(q_last, q - 2, q) % q
    return out


def rescale_wrong_inverse(p, acc):              # multiplies by q_last instead of its inverse
    q_last = p.primes[-1]
    r = np.asarray(acc, dtype=np.int64)[:, -1]
    r_c = np.where(r > (q_last - 1) // 2, r - q_last, r)
    out = np.zeros((2, p.n_limbs - 1, p.N), dtype=np.int64)
    for j, q in enumerate(p.primes[:-1]):
        out[:, j] = ((acc[:, j] - r_c) % q) * (q_last % q) % q
    return out


def _encrypt_variant(drop_e1=False, minus_m=False, swap_pk=False, shared_noise=False):
    def enc(p, keys, m, seed, client_id, ct_index):
        m = np.asarray(m, dtype=np.int64)
        u = philox.sample_ternary(seed, p.N, ct_index, client_id, philox.TAG_U)
        e0 = philox.sample_cbd(seed, p.N, p.cbd_eta, ct_index, client_id, philox.TAG_E0)
        e1 = philox.sample_cbd(seed, p.N, p.cbd_eta, ct_index, client_id, philox.TAG_E0 if shared_noise else philox.TAG_E1)
        ct = np.zeros((2, p.n_limbs, p.N), dtype=np.int64)
        for j, q in enumerate(p.primes):
            b, a = (keys.pk_a[j], keys.pk_b[j]) if swap_pk else (keys.pk_b[j], keys.pk_a[j])
            ct[0, j] = (ring.negacyclic_mul(b, u % q, q, p.psi(j)) + e0 + (-m if minus_m else m)) % q
            ct[1, j] = (ring.negacyclic_mul(a, u % q, q, p.psi(j)) + (0 if drop_e1 else e1)) % q
        return ct
    return enc


def keygen_wrong_sign(p, seed):                 # b = a*s + e instead of -a*s + e
    good = _GOOD["keygen"](p, seed)
    pk_b = np.stack([(2 * good.e - good.pk_b[j]) % q for j, q in enumerate(p.primes)])
    return scheme.KeyPair(s=good.s, pk_b=pk_b, pk_a=good.pk_a, e=good.e)


def weights_floor(p, alpha):                    # truncates instead of rounding to nearest
    return [int(x) for x in np.floor(np.asarray(alpha, dtype=np.float64) * np.float64(p.primes[-1]))]


def crt_not_centered(residues, primes):         # lift to [0, Q) instead of (-Q/2, Q/2]
    big_q = int(np.prod([int(q) for q in primes], dtype=object))
    return [v % big_q for v in _GOOD["crt_centered"](residues, primes)]


def intt_without_scaling(a_hat, q, psi):        # forgets the factor 1/N
    n_ring = len(a_hat)
    return (_GOOD["intt"](a_hat, q, psi) * n_ring) % q


def ntt_cyclic(a, q, psi):                      # cyclic transform: the powers of psi are not merged in
    a = np.asarray(a, dtype=np.int64)
    inv = pow(psi, q - 2, q)
    tw = np.array([pow(inv, i, q) for i in range(len(a))], dtype=object)
    return _GOOD["ntt"](np.array([int(x) for x in (a.astype(object) * tw) % q], dtype=np.int64), q, psi)


def ntt_natural_order(a, q, psi):               # evaluations in natural instead of bit-reversed order
    out = _GOOD["ntt"](a, q, psi)
    bits = len(out).bit_length() - 1
    return out[[ring.bit_reverse(i, bits) for i in range(len(out))]]


def ternary_wrong_word(seed, n_coeff, ct_index, client_id, tag):   # words of a block taken in reverse
    words = philox._blocks(seed, (n_coeff + 3) // 4, ct_index, client_id, tag)[:, ::-1].reshape(-1)[:n_coeff]
    return ((words.astype(np.uint64) * np.uint64(3)) >> np.uint64(32)).astype(np.int64) - 1


def cbd_wrong_mask(seed, n_coeff, eta, ct_index, client_id, tag):  # uses eta + 1 bits
    return _GOOD["sample_cbd"](seed, n_coeff, min(eta + 1, 32), ct_index, client_id, tag) if eta else _GOOD["sample_cbd"](seed, n_coeff, 0, ct_index, client_id, tag)


def uniform_low_word_only(seed, n_coeff, q, ct_index, client_id, tag):   # reduces one 32-bit word instead of 64 bits
    w = philox._blocks(seed, (n_coeff + 1) // 2, ct_index, client_id, tag).reshape(-1, 2)[:n_coeff]
    return (w[:, 0].astype(np.uint64) % np.uint64(q)).astype(np.int64)


def encode_sine(z, log2_n, scale_bits):         # sine instead of cosine
    n_ring = 1 << log2_n
    g = encoder.rotation_group(log2_n)
    k = np.arange(n_ring, dtype=np.int64).reshape(-1, 1)
    ang = np.pi * ((k * g.reshape(1, -1)) % (2 * n_ring)).astype(np.float64) / n_ring
    return np.rint((2.0 * float(1 << scale_bits) / n_ring) * (np.sin(ang) @ np.asarray(z, dtype=np.float64))).astype(np.int64)


def encode_missing_factor_two(z, log2_n, scale_bits):   # Delta/N instead of 2*Delta/N
    return _GOOD["encode_def"](np.asarray(z, dtype=np.float64) / 2, log2_n, scale_bits)


def encode_fft_natural_slots(z, log2_n, scale_bits):    # slot j placed at bin j instead of (5^j - 1)/4
    n_ring = 1 << log2_n
    n = n_ring // 2
    c = np.fft.fft(np.asarray(z, dtype=np.complex128)) / n
    c = c * np.exp(-1j * np.pi * np.arange(n) / n_ring) * float(1 << scale_bits)
    return np.rint(np.concatenate([c.real, c.imag])).astype(np.int64)


def decode_wrong_scale(v, log2_n, scale_bits):  # divides by 2*Delta
    return _GOOD["decode_def"](v, log2_n, scale_bits) / 2


def encode_fixed_scale(z, log2_n, scale_bits):  # ignores the scaling bits: always 2^30
    return _GOOD["encode_def"](z, log2_n, 30)


def decode_fft_fixed_scale(v, log2_n, scale_bits):      # the fast decoder divides by 2^30 whatever the scale
    return _GOOD["decode_fft"](v, log2_n, 30)


def decrypt_residues_without_c0(p, keys, ct, level):    # d = c1 * s
    zero = np.zeros_like(np.asarray(ct, dtype=np.int64))
    zero[1] = np.asarray(ct, dtype=np.int64)[1]
    return _GOOD["decrypt_residues"](p, keys, zero, level)


def decrypt_residues_minus(p, keys, ct, level):         # d = c0 - c1 * s
    ct = np.asarray(ct, dtype=np.int64).copy()
    for j in range(level):
        ct[1, j] = (-ct[1, j]) % p.primes[j]
    return _GOOD["decrypt_residues"](p, keys, ct, level)


def plain_fedavg_float32(ws, alpha):            # accumulates in float32
    acc = np.zeros(np.asarray(ws[0]).shape, dtype=np.float32)
    for a, w in zip(alpha, ws):
        acc = acc + np.float32(a) * np.asarray(w, dtype=np.float32)
    return acc


def plain_fedavg_unweighted(ws, alpha):         # drops the weights
    return (sum(np.asarray(w).astype(np.float64) for w in ws) / len(ws)).astype(np.float32)


def select_ties_to_higher_index(sens, ratio):
    s = np.asarray(sens, dtype=np.float32).astype(np.float64)
    k = select.select_count(s.shape[0], ratio)
    mask = np.zeros(s.shape[0], dtype=bool)
    if k > 0:
        mask[np.lexsort((-np.arange(s.shape[0]), -s))[:k]] = True
    return mask


def select_smallest(sens, ratio):               # keeps the least sensitive parameters
    return _GOOD["select_top"](-np.asarray(sens, dtype=np.float32), ratio)


_GOOD = {"keygen": scheme.keygen, "crt_centered": scheme.crt_centered, "intt": ring.intt, "ntt": ring.ntt,
         "sample_cbd": philox.sample_cbd, "encode_def": encoder.encode_def, "decode_def": encoder.decode_def,
         "decode_fft": encoder.decode_fft, "decrypt_residues": scheme.decrypt_residues,
         "select_top": select.select_top}


def _with_ctx(pin):
    return lambda: pin(_small_ctx())


CASES = [
    ("rescale rounds down", scheme, "rescale", rescale_floor, _with_ctx(pins_scheme.test_rescale_matches_big_integer_definition)),
    ("rescale multiplies by q_last", scheme, "rescale", rescale_wrong_inverse, _with_ctx(pins_scheme.test_rescale_matches_big_integer_definition)),
    ("encrypt drops e1", scheme, "encrypt", _encrypt_variant(drop_e1=True), _with_ctx(pins_scheme.test_encrypt_noise_identity)),
    ("encrypt subtracts m", scheme, "encrypt", _encrypt_variant(minus_m=True), _with_ctx(pins_scheme.test_encrypt_noise_identity)),
    ("encrypt swaps the key halves", scheme, "encrypt", _encrypt_variant(swap_pk=True), _with_ctx(pins_scheme.test_encrypt_noise_identity)),
    ("encrypt reuses e0's stream for e1", scheme, "encrypt", _encrypt_variant(shared_noise=True), _with_ctx(pins_scheme.test_encrypt_noise_identity)),
    ("keygen b = a*s + e", scheme, "keygen", keygen_wrong_sign, lambda: pins_scheme.test_keygen_relation((Params(6, 3), scheme.keygen(Params(6, 3), 5)))),
    ("weights truncated", scheme, "integer_weights", weights_floor, _with_ctx(pins_scheme.test_aggregate_is_homomorphic)),
    ("lift not centred", scheme, "crt_centered", crt_not_centered, pins_scheme.test_crt_lift_against_integers),
    ("inverse transform without 1/N", ring, "intt", intt_without_scaling, lambda: pins_ring.test_transform_equals_evaluation_and_product_equals_schoolbook(3)),
    ("cyclic instead of negacyclic transform", ring, "ntt", ntt_cyclic, lambda: pins_ring.test_transform_equals_evaluation_and_product_equals_schoolbook(3)),
    ("transform in natural order", ring, "ntt", ntt_natural_order, pins_ring.test_transform_output_order),
    ("Philox multipliers swapped", philox, "M0", philox.M1, pins_philox.test_philox_known_answers),
    ("Philox Weyl constant off by one", philox, "W0", philox.W0 + 1, pins_philox.test_philox_known_answers),
    ("ternary sampler reads the block backwards", philox, "sample_ternary", ternary_wrong_word, pins_philox.test_samplers_follow_their_word_layout),
    ("binomial sampler uses eta + 1 bits", philox, "sample_cbd", cbd_wrong_mask, pins_philox.test_samplers_follow_their_word_layout),
    ("uniform sampler reduces 32 bits", philox, "sample_uniform", uniform_low_word_only, pins_philox.test_samplers_follow_their_word_layout),
    ("encoder with sine", encoder, "encode_def", encode_sine, lambda: pins_encoder.test_encode_closed_forms(4, 30)),
    ("encoder without the factor 2", encoder, "encode_def", encode_missing_factor_two, lambda: pins_encoder.test_encode_closed_forms(4, 30)),
    ("fast encoder with slots at natural bins", encoder, "encode_fft", encode_fft_natural_slots, lambda: pins_encoder.test_encode_closed_forms(4, 30)),
    ("decoder divides by 2*Delta", encoder, "decode_def", decode_wrong_scale, lambda: pins_encoder.test_decode_is_evaluation_at_the_rotation_group(4, 30)),
    ("encoder ignores the scaling bits", encoder, "encode_def", encode_fixed_scale, lambda: pins_encoder.test_encode_closed_forms(4, 20)),
    ("fast decoder ignores the scaling bits", encoder, "decode_fft", decode_fft_fixed_scale, lambda: pins_encoder.test_decode_is_evaluation_at_the_rotation_group(4, 20)),
    ("decryption drops c0", scheme, "decrypt_residues", decrypt_residues_without_c0, _with_ctx(pins_scheme.test_decrypt_residues_per_limb)),
    ("decryption subtracts c1*s", scheme, "decrypt_residues", decrypt_residues_minus, _with_ctx(pins_scheme.test_decrypt_residues_per_limb)),
    ("plain FedAvg in float32", fedavg, "plain_fedavg", plain_fedavg_float32, pins_fedavg.test_plain_fedavg_against_exact_rationals),
    ("plain FedAvg ignores the weights", fedavg, "plain_fedavg", plain_fedavg_unweighted, pins_fedavg.test_plain_fedavg_against_exact_rationals),
    ("selection ties to the higher index", select, "select_top", select_ties_to_higher_index, pins_select.test_select_matches_the_counting_definition),
    ("selection of the least sensitive", select, "select_top", select_smallest, pins_select.test_select_closed_forms_and_rounding),
]


@pytest.mark.parametrize("name,module,attr,mutant,pin", CASES, ids=[c[0] for c in CASES])
def test_pin_rejects_planted_mistake(monkeypatch, name, module, attr, mutant, pin):
    monkeypatch.setattr(module, attr, mutant)
    ring._TABLES.clear()
    with pytest.raises(AssertionError):
        pin()


def test_pins_accept_the_unmodified_oracle():
    """The same calls pass without a planted mistake (so a rejection above is the mistake's doing)."""
    for _, _, _, _, pin in CASES:
        pin()
