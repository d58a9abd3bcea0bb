"""Pins for the oracle's scheme: algebraic invariants that do not go through its own code path twice."""
import numpy as np
import pytest

from oracle import encoder, fedavg, philox as rng, ring, scheme
from oracle.params import Params


def _centered(x, q):
    x = np.asarray(x, dtype=np.int64) % q
    return np.where(x > q // 2, x - q, x)


def _signed_negacyclic(a, b):
    """Exact integer negacyclic product of small signed vectors (no modulus)."""
    n_ring = len(a)
    full = np.convolve(np.asarray(a, dtype=np.int64), np.asarray(b, dtype=np.int64))
    full = np.concatenate([full, [0]])
    return full[:n_ring] - full[n_ring:]


@pytest.fixture(scope="module", params=[(6, 3), (13, 3), (14, 4)])
def ctx(request):
    log2_n, limbs = request.param
    p = Params(log2_n, limbs)
    return p, scheme.keygen(p, 0xC0FFEE + log2_n)


def test_keygen_relation(ctx):
    p, keys = ctx
    assert set(np.unique(keys.s)) <= {-1, 0, 1} and np.abs(keys.e).max() <= p.cbd_eta
    for j, q in enumerate(p.primes):
        lhs = (keys.pk_b[j] + ring.negacyclic_mul_def(keys.pk_a[j], keys.s % q, q)) % q
        assert np.array_equal(_centered(lhs, q), keys.e)         # b + a*s = e, small
        assert keys.pk_a[j].min() >= 0 and keys.pk_a[j].max() < q
    # the public polynomial a differs per limb (independent streams), s is shared
    assert not np.array_equal(keys.pk_a[0] % p.primes[1], keys.pk_a[1])


def test_encrypt_noise_identity(ctx):
    """c0 + c1*s - m == e_pk*u + e0 + e1*s exactly, the right side built from the sampled pieces."""
    p, keys = ctx
    seed, client, ct_index = 424242, 2, 5
    rs = np.random.default_rng(3)
    m = rs.integers(-(1 << 28), 1 << 28, p.N)
    ct = scheme.encrypt(p, keys, m, seed, client, ct_index)
    u = rng.sample_ternary(seed, p.N, ct_index, client, rng.TAG_U)
    e0 = rng.sample_cbd(seed, p.N, p.cbd_eta, ct_index, client, rng.TAG_E0)
    e1 = rng.sample_cbd(seed, p.N, p.cbd_eta, ct_index, client, rng.TAG_E1)
    noise = _signed_negacyclic(keys.e, u) + e0 + _signed_negacyclic(e1, keys.s)
    for j, q in enumerate(p.primes):
        lhs = (ct[0, j] + ring.negacyclic_mul_def(ct[1, j], keys.s % q, q) - m) % q
        assert np.array_equal(_centered(lhs, q), noise)
    assert ct.min() >= 0 and all(ct[:, j].max() < q for j, q in enumerate(p.primes))
    # decrypt(encrypt(m)) = m + noise, and the noise has the predicted size
    v = np.array(scheme.decrypt(p, keys, ct, p.n_limbs), dtype=object)
    assert np.array_equal(np.array([int(x) for x in v - m.astype(object)]), noise)
    if p.N >= 8192:
        pred = np.sqrt(p.cbd_eta / 2 * (2 / 3) * p.N * 2 + p.cbd_eta / 2)
        assert 0.9 * pred < noise.std() < 1.1 * pred
    # a different ciphertext index or client gives different randomness
    assert not np.array_equal(ct, scheme.encrypt(p, keys, m, seed, client, ct_index + 1))
    assert not np.array_equal(ct, scheme.encrypt(p, keys, m, seed, client + 1, ct_index))


def test_crt_lift_against_integers():
    primes = (2147352577, 2146959361, 2146336769)
    big_q = primes[0] * primes[1] * primes[2]
    vals = [0, 1, -1, big_q // 2, -(big_q // 2), 123456789012345678901234, -98765432109876543210]
    res = np.array([[v % q for v in vals] for q in primes], dtype=np.int64)
    assert scheme.crt_centered(res, primes) == vals


def test_rescale_matches_big_integer_definition(ctx):
    p, _ = ctx
    rs = np.random.default_rng(8)
    acc = np.stack([rs.integers(0, q, (2, p.N)) for q in p.primes], axis=1)
    out = scheme.rescale(p, acc)
    q_last = p.primes[-1]
    for poly in range(2):
        x = scheme.crt_centered(acc[poly], p.primes)                 # integer represented by all L limbs
        for k in range(0, p.N, max(1, p.N // 64)):
            r = x[k] % q_last
            r_c = r - q_last if r > (q_last - 1) // 2 else r
            y = (x[k] - r_c) // q_last
            assert (x[k] - r_c) % q_last == 0 and abs(y * q_last - x[k]) <= q_last // 2
            for j, q in enumerate(p.primes[:-1]):
                assert out[poly, j, k] == y % q


def test_aggregate_is_homomorphic(ctx):
    """decrypt(weighted sum) == sum_i w_i * (m_i + noise_i) over the integers (mod Q, centred)."""
    p, keys = ctx
    rs = np.random.default_rng(21)
    K = 4
    counts = rs.integers(100, 1001, K)
    alpha = counts / counts.sum()
    w = scheme.integer_weights(p, alpha)
    assert w == [round(float(a) * p.primes[-1]) for a in alpha] and abs(sum(w) - p.primes[-1]) <= K
    ms = [rs.integers(-(1 << 27), 1 << 27, p.N) for _ in range(K)]
    cts = [scheme.encrypt(p, keys, m, 77, i, 0) for i, m in enumerate(ms)]
    plain = [np.array(scheme.decrypt(p, keys, ct, p.n_limbs), dtype=object) for ct in cts]
    expect = sum(wi * pl for wi, pl in zip(w, plain))
    acc = scheme.weighted_sum(p, cts, alpha)
    got = np.array(scheme.decrypt(p, keys, acc, p.n_limbs), dtype=object)
    assert np.array_equal(got, expect)             # |expect| << Q/2, so no wrap
    # after the rescale the plaintext is expect / q_last up to the rounding terms tau0 + tau1*s
    out = scheme.aggregate(p, cts, alpha)
    dec = np.array(scheme.decrypt(p, keys, out, p.n_limbs - 1), dtype=object)
    bound = (1 + np.abs(keys.s).sum()) / 2 + 1
    diff = dec * p.primes[-1] - expect
    assert max(abs(int(d)) for d in diff) <= bound * p.primes[-1]


def test_single_client_unit_weight_is_identity(ctx):
    p, keys = ctx
    m = np.random.default_rng(2).integers(-(1 << 28), 1 << 28, p.N)
    ct = scheme.encrypt(p, keys, m, 5, 0, 0)
    assert scheme.integer_weights(p, [1.0]) == [p.primes[-1]]
    out = scheme.aggregate(p, [ct], [1.0])
    assert np.array_equal(out, ct[:, :-1])


@pytest.mark.parametrize("log2_n,limbs,K,std", [(13, 3, 3, 0.05), (14, 4, 8, 0.02)])
def test_round_against_float64_fedavg(log2_n, limbs, K, std):
    p = Params(log2_n, limbs)
    keys = scheme.keygen(p, 99)
    rs = np.random.default_rng(4)
    P = 3 * p.n_slots + 1234
    ws = [rs.normal(0, std, P).astype(np.float32) for _ in range(K)]
    counts = rs.integers(100, 1001, K)
    alpha = counts / counts.sum()
    runs = [(10, 2 * p.n_slots), (2 * p.n_slots + 500, 777)]
    out = fedavg.secure_round(p, keys, ws, alpha, runs, seed=31337)
    ref = fedavg.fedavg_float64(ws, alpha)
    enc_idx, plain_idx = fedavg.mask_indices(P, runs)
    assert np.array_equal(out[plain_idx], ref[plain_idx].astype(np.float32))
    err = out[enc_idx].astype(np.float64) - ref[enc_idx]
    sigma = fedavg.noise_sigma(p, alpha)
    rms = float(np.sqrt((err ** 2).mean()))
    # RMS follows the noise model; the maximum gets a wide bound because a slot's noise is
    # e_pk(zeta_j)*sum_i alpha_i u_i(zeta_j) + ...: a Gaussian whose variance is itself random per slot
    # (|e_pk(zeta_j)|^2 is exponential), i.e. Laplace-like tails, P(|x| > t*sigma) ~ exp(-1.41 t).
    assert 0.7 * sigma < rms < 1.4 * sigma and np.abs(err).max() < 16 * sigma
    # dropout: aggregating a subset with renormalised weights equals FedAvg over the subset
    sub = [0, 2]
    a_sub = alpha[sub] / alpha[sub].sum()
    out_sub = fedavg.secure_round(p, keys, [ws[i] for i in sub], a_sub, runs, seed=31337)
    ref_sub = fedavg.fedavg_float64([ws[i] for i in sub], a_sub)
    assert np.abs(out_sub[enc_idx] - ref_sub[enc_idx]).max() < 16 * fedavg.noise_sigma(p, a_sub)


def test_noiseless_mode_is_tight():
    """eta = 0: only encode rounding, weight rounding and rescale rounding remain."""
    p = Params(13, 3, cbd_eta=0)
    keys = scheme.keygen(p, 1)
    rs = np.random.default_rng(6)
    K, P = 3, p.n_slots
    ws = [rs.normal(0, 0.05, P).astype(np.float32) for _ in range(K)]
    alpha = np.array([0.2, 0.3, 0.5])
    out = fedavg.secure_round(p, keys, ws, alpha, [(0, P)], seed=2)
    ref = fedavg.fedavg_float64(ws, alpha)
    # rescale rounding tau0 + tau1*s: sigma about sqrt(N * (1 + 2N/3) / 24) / Delta = 2.5e-6 at N = 8192... per slot
    sig = np.sqrt(p.N * (1 + 2 * p.N / 3) / 24.0) / p.delta
    err = out.astype(np.float64) - ref
    assert np.abs(err).max() < 8 * sig + 2 ** -24 * 0.3 and np.sqrt((err ** 2).mean()) < 1.5 * sig + 2e-8


# ---- variant: weighing on the client, the server only adds (Section "Comparison with Other FL Frameworks") ----

def test_ciphertext_sum_is_the_sum_of_plaintexts(ctx):
    """Decrypting the sum gives exactly the sum of what each ciphertext decrypts to (no wrap: << Q/2)."""
    p, keys = ctx
    rs = np.random.default_rng(11)
    K = 5
    ms = [rs.integers(-(1 << 27), 1 << 27, p.N) for _ in range(K)]
    cts = [scheme.encrypt(p, keys, m, 123, i, 3) for i, m in enumerate(ms)]
    each = [np.array(scheme.decrypt(p, keys, ct, p.n_limbs), dtype=object) for ct in cts]
    got = np.array(scheme.decrypt(p, keys, scheme.sum_ciphertexts(p, cts), p.n_limbs), dtype=object)
    assert np.array_equal(got, sum(each))
    # one client: the sum is the ciphertext itself
    assert np.array_equal(scheme.sum_ciphertexts(p, [cts[0]]), cts[0])
    # residues stay canonical even for the largest inputs
    big = np.stack([np.stack([np.full(p.N, q - 1, dtype=np.int64) for q in p.primes])] * 2)
    s3 = scheme.sum_ciphertexts(p, [big, big, big])
    for j, q in enumerate(p.primes):
        assert np.all(s3[:, j] == (3 * (q - 1)) % q)


@pytest.mark.parametrize("log2_n,limbs,K,std", [(13, 2, 3, 0.05), (14, 3, 8, 0.02)])
def test_client_weighted_round_against_float64_fedavg(log2_n, limbs, K, std):
    p = Params(log2_n, limbs)
    keys = scheme.keygen(p, 99)
    rs = np.random.default_rng(4)
    P = 3 * p.n_slots + 1234
    ws = [rs.normal(0, std, P).astype(np.float32) for _ in range(K)]
    counts = rs.integers(100, 1001, K)
    alpha = counts / counts.sum()
    runs = [(10, 2 * p.n_slots), (2 * p.n_slots + 500, 777)]
    out = fedavg.secure_round_client_weighted(p, keys, ws, alpha, runs, seed=31337)
    ref = fedavg.fedavg_float64(ws, alpha)
    enc_idx, plain_idx = fedavg.mask_indices(P, runs)
    # plaintext part: every client rounds alpha*w to float32 first, so it matches FedAvg to float32 accuracy only
    assert np.abs(out[plain_idx].astype(np.float64) - ref[plain_idx]).max() < K * 2.0 ** -24 * np.abs(ref[plain_idx]).max() + 1e-9
    err = out[enc_idx].astype(np.float64) - ref[enc_idx]
    sigma = fedavg.noise_sigma_client_weighted(p, K)
    rms = float(np.sqrt((err ** 2).mean()))
    assert 0.7 * sigma < rms < 1.4 * sigma and np.abs(err).max() < 16 * sigma
    # the K unweighted noises make this variant noisier than weighing on the server
    assert sigma > 1.5 * fedavg.noise_sigma(Params(log2_n, limbs + 1), alpha)


def test_client_weighted_plain_part_exact_cases():
    w = np.array([0.1, -0.25, 3.0, 1e-8], dtype=np.float32)
    assert np.array_equal(fedavg.plain_weighted(w, 1.0), w)
    assert np.array_equal(fedavg.plain_weighted(w, 0.5), (w.astype(np.float64) / 2).astype(np.float32))
    assert np.array_equal(fedavg.plain_sum([w, w]), (2 * w.astype(np.float64)).astype(np.float32))


def test_decrypt_residues_per_limb(ctx):
    """The residues before the lift: in every limb d_j - m is the fresh noise built from the sampled pieces (reduced
    mod q_j), at the full level and with the last limb dropped; lifting them gives what decrypt returns."""
    p, keys = ctx
    seed, client, ct_index = 777, 1, 9
    rs = np.random.default_rng(5)
    m = rs.integers(-(1 << 28), 1 << 28, p.N)
    ct = scheme.encrypt(p, keys, m, seed, client, ct_index)
    u = rng.sample_ternary(seed, p.N, ct_index, client, rng.TAG_U)
    e0 = rng.sample_cbd(seed, p.N, p.cbd_eta, ct_index, client, rng.TAG_E0)
    e1 = rng.sample_cbd(seed, p.N, p.cbd_eta, ct_index, client, rng.TAG_E1)
    noise = _signed_negacyclic(keys.e, u) + e0 + _signed_negacyclic(e1, keys.s)
    for level in (p.n_limbs, p.n_limbs - 1, 1):
        d = scheme.decrypt_residues(p, keys, ct[:, :level], level)
        assert d.shape == (level, p.N) and d.min() >= 0
        for j in range(level):
            q = p.primes[j]
            assert d[j].max() < q
            assert np.array_equal(_centered(d[j] - m, q), noise)
        assert scheme.crt_centered(d, p.primes[:level]) == scheme.decrypt(p, keys, ct[:, :level], level)
        if level > 1:      # one limb alone cannot hold m + noise centred (|m| reaches 2^28 < q/2: it can), more limbs agree
            assert scheme.decrypt(p, keys, ct[:, :level], level) == [int(x) for x in (m + noise)]


def test_reusing_a_seed_leaks_the_update_difference(ctx):
    """Why (seed, client) must be fresh for every round: with the same randomness the two ciphertexts share c1, and
    c0 - c0' is the difference of the plaintexts, readable without any key."""
    p, keys = ctx
    rs = np.random.default_rng(6)
    m1 = rs.integers(-(1 << 28), 1 << 28, p.N)
    m2 = rs.integers(-(1 << 28), 1 << 28, p.N)
    a = scheme.encrypt(p, keys, m1, 99, 3, 0)
    b = scheme.encrypt(p, keys, m2, 99, 3, 0)
    assert np.array_equal(a[1], b[1])
    for j, q in enumerate(p.primes):
        assert np.array_equal(_centered(a[0, j] - b[0, j], q), m1 - m2)
    c = scheme.encrypt(p, keys, m2, 100, 3, 0)          # a fresh seed: nothing in common
    assert not np.array_equal(a[1], c[1])
    assert not np.array_equal(_centered(a[0, 0] - c[0, 0], p.primes[0]), m1 - m2)


@pytest.mark.parametrize("log2_n,limbs,scale_bits", [(11, 3, 20), (13, 3, 20), (11, 3, 30)])
def test_round_at_other_crypto_parameters(log2_n, limbs, scale_bits):
    """The crypto-parameter sweep's settings (packing batch 1024 and 4096, 20 scaling bits): the whole oracle round
    against float64 FedAvg under the noise model, whose sigma scales with 1 / Delta."""
    p = Params(log2_n, limbs, scale_bits=scale_bits)
    keys = scheme.keygen(p, 4321)
    rs = np.random.default_rng(14)
    K = 3
    P = 2 * p.n_slots + 321
    ws = [rs.normal(0, 0.05, P).astype(np.float32) for _ in range(K)]
    alpha = np.array([0.5, 0.3, 0.2])
    runs = [(7, p.n_slots + 11), (p.n_slots + 100, p.n_slots // 2)]
    out = fedavg.secure_round(p, keys, ws, alpha, runs, seed=5)
    out_def = fedavg.secure_round(p, keys, ws, alpha, runs, seed=5, fast=False) if log2_n <= 11 else None
    ref = fedavg.fedavg_float64(ws, alpha)
    enc_idx, plain_idx = fedavg.mask_indices(P, runs)
    assert np.array_equal(out[plain_idx], ref[plain_idx].astype(np.float32))
    err = out[enc_idx].astype(np.float64) - ref[enc_idx]
    sigma = fedavg.noise_sigma(p, alpha)
    assert sigma == pytest.approx(fedavg.noise_sigma(Params(log2_n, limbs), alpha) * 2.0 ** (30 - scale_bits))
    assert 0.7 * sigma < np.sqrt((err ** 2).mean()) < 1.4 * sigma and np.abs(err).max() < 16 * sigma
    if out_def is not None:     # the definition-based encoder / decoder give the same round up to the encoder's +-1
        assert np.abs(out_def.astype(np.float64) - out.astype(np.float64)).max() <= 4.0 * p.N ** 0.5 / p.delta + 1e-7
