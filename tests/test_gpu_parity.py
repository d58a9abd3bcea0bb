"""GPU parity: every step of the HIP path against the CPU oracle, through the C ABI.

Integer ring work is compared bit for bit; encoded coefficients within +-1; decoded values
within 1e-6 absolute (the tolerance the benchmark spec states for the decoded aggregate; both sides
decode the same integers, so the real difference is rounding-order noise around 1e-12).
"""
import numpy as np
import pytest
import torch

from oracle import encoder as oenc
from oracle import fedavg as ofed
from oracle import ring as oring
from oracle import scheme as osch
from oracle.params import Params

pytestmark = pytest.mark.gpu

SEED = 0x5EED1234ABCD


@pytest.fixture(scope="module")
def he():
    from paper_2303_10837_amd import binding
    binding.load()
    torch.cuda.set_device(0)
    return binding


def _np(t):
    return t.detach().cpu().numpy()


def _dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


_CTX_CACHE = {}


def _setup(he, log2_n, limbs, eta=21):
    key = (log2_n, limbs, eta)
    if key not in _CTX_CACHE:
        ctx = he.Context(log2_n, limbs, cbd_eta=eta)
        keys = he.he_keygen(ctx, SEED)
        p = Params(log2_n, limbs, cbd_eta=eta)
        okeys = osch.keygen(p, SEED)
        _CTX_CACHE[key] = (ctx, keys, p, okeys)
    return _CTX_CACHE[key]


@pytest.mark.parametrize("log2_n,limbs", [(3, 3), (4, 3), (5, 2), (6, 3), (7, 3), (9, 3), (10, 3), (11, 3), (12, 3), (12, 8), (13, 3), (14, 4)])
def test_context_and_transform(he, log2_n, limbs):
    ctx, _, p, _ = _setup(he, log2_n, limbs)
    assert ctx.primes == p.primes and ctx.N == p.N
    rs = np.random.default_rng(log2_n)
    for j, q in enumerate(p.primes):
        polys = np.stack([rs.integers(0, q, p.N), np.full(p.N, q - 1), np.arange(p.N) % q,
                          rs.integers(0, q, p.N), np.zeros(p.N, dtype=np.int64)]).astype(np.int64)
        d = _dev(polys, torch.int32)
        he.he_debug_ntt(ctx, False, j, d)
        fwd = _np(d).astype(np.int64)
        for b in range(polys.shape[0]):
            assert np.array_equal(fwd[b], oring.ntt(polys[b], q, p.psi(j))), (log2_n, j, b)
        he.he_debug_ntt(ctx, True, j, d)
        assert np.array_equal(_np(d).astype(np.int64), polys)


def _boundary_values(rs, q, shape):
    """Residues at the edges of the lazy ranges the kernels keep: 0, 1, q-1, q-2, (q-1)/2, (q+1)/2, mixed at random
    with a few ordinary values."""
    edge = np.array([0, 1, q - 1, q - 2, (q - 1) // 2, (q + 1) // 2, 2, q - 3], dtype=np.int64)
    v = edge[rs.integers(0, len(edge), shape)]
    ordinary = rs.random(shape) < 0.1
    v[ordinary] = rs.integers(0, q, int(ordinary.sum()))
    return v


@pytest.mark.parametrize("log2_n,limbs", [(10, 3), (11, 3), (12, 4), (13, 3), (14, 4)])
def test_transform_and_decrypt_on_boundary_values(he, log2_n, limbs):
    """Inputs made of the extreme residues (every butterfly sees sums and differences at the edges of [0, q) and
    [0, 2q)): the transforms, and decryption of ciphertexts made of such residues, stay bit-exact."""
    ctx, keys, p, okeys = _setup(he, log2_n, limbs)
    rs = np.random.default_rng(100 + log2_n)
    for j, q in enumerate(p.primes):
        polys = _boundary_values(rs, q, (12, p.N))
        d = _dev(polys, torch.int32)
        he.he_debug_ntt(ctx, False, j, d)
        fwd = _np(d).astype(np.int64)
        for b in range(polys.shape[0]):
            assert np.array_equal(fwd[b], oring.ntt(polys[b], q, p.psi(j))), (log2_n, j, b)
        he.he_debug_ntt(ctx, True, j, d)
        assert np.array_equal(_np(d).astype(np.int64), polys)
        # inverse first, from boundary values in the evaluation domain
        d = _dev(polys, torch.int32)
        he.he_debug_ntt(ctx, True, j, d)
        inv = _np(d).astype(np.int64)
        for b in range(0, polys.shape[0], 4):
            assert np.array_equal(inv[b], oring.intt(polys[b], q, p.psi(j))), (log2_n, j, b)
    cts = np.stack([_boundary_values(rs, q, (3, 2, p.N)) for q in p.primes], axis=2)
    for lvl in (limbs - 1, limbs):
        got = _np(he.he_debug_decrypt_residues(ctx, keys, _dev(cts[:, :, :lvl], torch.int32), lvl)).astype(np.int64)
        for c in range(cts.shape[0]):
            assert np.array_equal(got[c], osch.decrypt_residues(p, okeys, cts[c][:, :lvl], lvl)), (log2_n, lvl, c)
    # aggregation of such ciphertexts with weights at the ends of their range
    K = 5
    alpha = np.array([1e-6, 0.5, 0.25, 0.2, 1.0 - 0.95 - 1e-6])
    ins = [np.stack([_boundary_values(rs, q, (2, 2, p.N)) for q in p.primes], axis=2) for _ in range(K)]
    out, _ = he.he_aggregate(ctx, alpha, [_dev(x, torch.int32) for x in ins], [None] * K)
    out = _np(out).astype(np.int64)
    for c in range(2):
        assert np.array_equal(out[c], osch.aggregate(p, [x[c] for x in ins], alpha)), (log2_n, c)


@pytest.mark.parametrize("log2_n,limbs", [(4, 3), (10, 3), (11, 2), (12, 3), (13, 3), (14, 4)])
def test_keygen(he, log2_n, limbs):
    ctx, keys, p, okeys = _setup(he, log2_n, limbs)
    pk, sk = he.he_debug_export_keys(ctx, keys)
    pk = _np(pk).astype(np.int64)
    assert np.array_equal(_np(sk).astype(np.int64), okeys.s)
    assert np.array_equal(pk[0], okeys.pk_b) and np.array_equal(pk[1], okeys.pk_a)


@pytest.mark.parametrize("log2_n,limbs", [(4, 3), (8, 3), (11, 3), (12, 3), (13, 3), (14, 4)])
def test_encode(he, log2_n, limbs):
    ctx, _, p, _ = _setup(he, log2_n, limbs)
    rs = np.random.default_rng(1)
    n = p.n_slots
    slots = rs.normal(0, 0.05, (5, n)).astype(np.float32)
    slots[1] = 0.3125                       # constant -> (Delta * c, 0, ..., 0)
    slots[2] = 0
    slots[2, min(3, n - 1)] = 1.0           # unit vector
    slots[3] = 0
    m = _np(he.he_debug_encode(ctx, _dev(slots))).astype(np.int64)
    assert m[1, 0] == int(0.3125 * 2 ** 30) and np.all(m[1, 1:] == 0)
    assert np.all(m[3] == 0)
    for c in range(5):
        ref = oenc.encode_fft(slots[c].astype(np.float64), log2_n, 30)
        diff = np.abs(m[c] - ref)
        assert diff.max() <= 1 and (diff != 0).mean() < 1e-3
        if log2_n <= 8:
            assert np.abs(m[c] - oenc.encode_def(slots[c].astype(np.float64), log2_n, 30)).max() <= 1


@pytest.mark.parametrize("log2_n,limbs,eta", [(4, 3, 21), (10, 3, 21), (11, 3, 21), (12, 5, 21), (13, 3, 21), (14, 4, 21), (13, 3, 0), (10, 2, 32), (12, 2, 32)])
def test_encrypt_given_plaintext(he, log2_n, limbs, eta):
    ctx, keys, p, okeys = _setup(he, log2_n, limbs, eta)
    rs = np.random.default_rng(2)
    n_ct, first, client = 3, 7, 5
    m = rs.integers(-(1 << 29), 1 << 29, (n_ct, p.N)).astype(np.int32)
    m[1, :8] = [2 ** 31 - 33, -(2 ** 31 - 33), 0, -1, 1, 2 ** 30, -2 ** 30, 12345]   # extreme plaintext values (m + e0 must fit int32)
    ct = _np(he.he_debug_encrypt_plain(ctx, keys, SEED + 1, client, first, _dev(m))).astype(np.int64)
    for c in range(n_ct):
        ref = osch.encrypt(p, okeys, m[c].astype(np.int64), SEED + 1, client, first + c)
        assert np.array_equal(ct[c], ref), (c,)


@pytest.mark.parametrize("log2_n,limbs", [(13, 3), (12, 2), (14, 5)])
def test_encrypt_ciphertext_counts_around_the_launch_grouping(he, log2_n, limbs):
    """The encryption kernel's grid comes in groups of 8 ciphertexts (one per XCD) x L limbs, with the surplus workgroups
    leaving at once: every count around those groups gives the same ciphertexts as the oracle."""
    ctx, keys, p, okeys = _setup(he, log2_n, limbs)
    rs = np.random.default_rng(11)
    m_all = rs.integers(-(1 << 29), 1 << 29, (17, p.N)).astype(np.int32)
    ref = {}
    for n_ct in (1, 7, 8, 9, 16, 17):
        ct = _np(he.he_debug_encrypt_plain(ctx, keys, SEED + 2, 3, 0, _dev(m_all[:n_ct]))).astype(np.int64)
        assert ct.shape[0] == n_ct
        for c in sorted({0, n_ct - 1, n_ct // 2}):
            if c not in ref:
                ref[c] = osch.encrypt(p, okeys, m_all[c].astype(np.int64), SEED + 2, 3, c)
            assert np.array_equal(ct[c], ref[c]), (n_ct, c)


@pytest.mark.parametrize("log2_n,limbs,K", [(4, 3, 3), (10, 2, 5), (13, 3, 3), (14, 4, 8), (10, 3, 1), (10, 3, 37), (10, 4, 70), (10, 3, 200),
                                            (10, 5, 70), (10, 8, 70), (13, 5, 9), (14, 8, 3), (10, 6, 130), (10, 3, 64), (10, 3, 65), (11, 5, 129)])
def test_aggregate_and_streaming(he, log2_n, limbs, K):
    ctx, _, p, _ = _setup(he, log2_n, limbs)
    rs = np.random.default_rng(3)
    n_ct, n_plain = 3, 100_003
    counts = rs.integers(100, 1001, K)
    alpha = counts / counts.sum()
    cts = [np.stack([rs.integers(0, q, (n_ct, 2, p.N)) for q in p.primes], axis=2).astype(np.int64) for _ in range(K)]
    cts[0][0, :, :, :4] = np.array(p.primes)[None, :, None] - 1          # largest residues
    plains = [rs.normal(0, 0.02, n_plain).astype(np.float32) for _ in range(K)]
    d_cts = [_dev(c, torch.int32) for c in cts]
    d_pl = [_dev(x) for x in plains]
    ct_g, pl_g = he.he_aggregate(ctx, alpha, d_cts, d_pl)
    ct_g = _np(ct_g).astype(np.int64)
    for c in range(n_ct):
        assert np.array_equal(ct_g[c], osch.aggregate(p, [x[c] for x in cts], alpha))
    assert np.array_equal(_np(pl_g), ofed.plain_fedavg(plains, alpha))
    # streaming form, uneven chunks, same client order -> identical bytes
    acc_ct, acc_pl = he.he_aggregate_begin(ctx, n_ct, n_plain)
    cut = max(1, K // 3)
    cut2 = min(K, cut + max(1, K // 7))
    for lo, hi in [(0, cut), (cut, cut2), (cut2, K)]:
        if hi > lo:
            he.he_aggregate_add(ctx, alpha[lo:hi], d_cts[lo:hi], d_pl[lo:hi], acc_ct, acc_pl)
    ct_s, pl_s = he.he_aggregate_finalize(ctx, acc_ct, acc_pl)
    assert torch.equal(ct_s.cpu(), torch.from_numpy(ct_g).to(torch.int32)) and torch.equal(pl_s, pl_g)
    # the accumulator before the rescale is the plain weighted sum of residues
    acc = _np(acc_ct).astype(np.int64)
    assert np.array_equal(acc[1], osch.weighted_sum(p, [x[1] for x in cts], alpha))
    # the same folds with the first one writing the accumulators (never zeroed: they start as garbage) and the last one
    # writing the outputs -> identical bytes again
    if K >= 2:
        acc_ct2 = torch.full_like(acc_ct, 0x5A5A5A5A)
        acc_pl2 = torch.full_like(acc_pl, float("nan"))
        chunks = [(lo, hi) for lo, hi in [(0, cut), (cut, cut2), (cut2, K)] if hi > lo]
        lo, hi = chunks[0]
        he.he_aggregate_add_first(ctx, alpha[lo:hi], d_cts[lo:hi], d_pl[lo:hi], acc_ct2, acc_pl2)
        for lo, hi in chunks[1:-1]:
            he.he_aggregate_add(ctx, alpha[lo:hi], d_cts[lo:hi], d_pl[lo:hi], acc_ct2, acc_pl2)
        lo, hi = chunks[-1]
        ct_f, pl_f = he.he_aggregate_add_last(ctx, alpha[lo:hi], d_cts[lo:hi], d_pl[lo:hi], acc_ct2, acc_pl2)
        assert torch.equal(ct_f, ct_s) and torch.equal(pl_f, pl_g)


def test_aggregate_special_cases(he):
    ctx, keys, p, okeys = _setup(he, 10, 3)
    rs = np.random.default_rng(4)
    ct = np.stack([rs.integers(0, q, (2, 2, p.N)) for q in p.primes], axis=2).astype(np.int64)
    d = _dev(ct, torch.int32)
    # one client, unit weight: the ciphertext comes back with its last limb dropped
    out, _ = he.he_aggregate(ctx, [1.0], [d], [None])
    assert np.array_equal(_np(out).astype(np.int64), ct[:, :, :-1])
    # only a plaintext part
    pl = [_dev(rs.normal(0, 1, 17).astype(np.float32)) for _ in range(2)]
    _, g = he.he_aggregate(ctx, [0.25, 0.75], [None, None], pl)
    assert np.array_equal(_np(g), ofed.plain_fedavg([_np(x) for x in pl], [0.25, 0.75]))
    # invalid weights are refused
    for bad in ([0.5, 0.6], [1.5, -0.5], [1e-12, 1.0 - 1e-12]):
        with pytest.raises(he.HeError):
            he.he_aggregate(ctx, bad, [d, d], [None, None])
    # ... by the streaming folds too (their weights need not sum to 1, but each must be a usable weight)
    acc_ct, acc_pl = he.he_aggregate_begin(ctx, 2, 0)
    for fold in (he.he_aggregate_add, he.he_aggregate_add_first, he.he_aggregate_add_last):
        with pytest.raises(he.HeError):
            fold(ctx, [0.5, -0.25], [d, d], [None, None], acc_ct, acc_pl)
        with pytest.raises(he.HeError):
            fold(ctx, [0.5, 1e-12], [d, d], [None, None], acc_ct, acc_pl)
    # two clients through first + last only (no begin, no middle fold, no finalize)
    he.he_aggregate_add_first(ctx, [0.25], [d], [None], acc_ct, acc_pl)
    out2, _ = he.he_aggregate_add_last(ctx, [0.75], [d], [None], acc_ct, acc_pl)
    ref2, _ = he.he_aggregate(ctx, [0.25, 0.75], [d, d], [None, None])
    assert torch.equal(out2, ref2)


@pytest.mark.parametrize("log2_n,limbs", [(4, 3), (10, 3), (11, 3), (12, 3), (13, 3), (14, 4), (10, 2)])
def test_decrypt_residues_and_decode(he, log2_n, limbs):
    ctx, keys, p, okeys = _setup(he, log2_n, limbs)
    rs = np.random.default_rng(5)
    level = limbs - 1
    m = rs.integers(-(1 << 29), 1 << 29, (2, p.N))
    cts = np.stack([osch.encrypt(p, okeys, m[c], SEED, 1, c) for c in range(2)])
    for lvl in (level, limbs):
        d = _np(he.he_debug_decrypt_residues(ctx, keys, _dev(cts[:, :, :lvl], torch.int32), lvl)).astype(np.int64)
        for c in range(2):
            assert np.array_equal(d[c], osch.decrypt_residues(p, okeys, cts[c][:, :lvl], lvl))
    # decode: arbitrary residues (full-range values exercise the centring), then realistic ones
    d_rand = np.stack([rs.integers(0, q, (2, p.N)) for q in p.primes[:level]], axis=1).astype(np.int64)
    d_real = np.stack([osch.decrypt_residues(p, okeys, cts[c][:, :level], level) for c in range(2)])
    for d in (d_rand, d_real):
        z = _np(he.he_debug_decode(ctx, _dev(d, torch.int32), level))
        for c in range(2):
            v = osch.crt_centered(d[c], p.primes[:level])
            ref = oenc.decode_fft(np.array([float(x) for x in v]), log2_n, 30)
            scale = max(1.0, np.abs(ref).max())
            assert np.abs(z[c] - ref).max() <= 1e-6 * scale if d is d_rand else np.abs(z[c] - ref).max() <= 1e-9


def test_decrypt_residues_beyond_one_launch(he):
    """More ciphertexts than one launch's grid takes (65535 in its second dimension): the call goes chunk by chunk."""
    ctx, keys, p, okeys = _setup(he, 11, 2)
    n_ct = 65536 + 5
    g = torch.Generator(device="cuda").manual_seed(3)
    ct = torch.stack([torch.randint(0, q, (n_ct, 2, p.N), generator=g, device="cuda", dtype=torch.int32) for q in p.primes], dim=2).contiguous()
    d = he.he_debug_decrypt_residues(ctx, keys, ct, 2)
    assert d.shape == (n_ct, 2, p.N)
    for c in (0, 32767, 32768, 65534, 65535, 65536, n_ct - 1):
        ref = osch.decrypt_residues(p, okeys, ct[c].cpu().numpy().astype(np.int64), 2)
        assert np.array_equal(d[c].cpu().numpy().astype(np.int64), ref), c


@pytest.mark.parametrize("log2_n,limbs", [(10, 3), (13, 3), (14, 4), (12, 5)])
def test_decrypt_merge_at_every_level(he, log2_n, limbs):
    """he_decrypt_merge_level at levels 1 .. L (a fresh ciphertext cut down to its first `level` limbs still decrypts to
    m + noise as long as that fits q_0 / 2): decoded and scattered values against the oracle's at the same level."""
    ctx, keys, p, okeys = _setup(he, log2_n, limbs)
    n = p.n_slots
    P = n + 37
    runs = [(3, n // 2), (n // 2 + 20, n // 2 + 5)]          # two ciphertexts, the second nearly empty
    mask = he.he_mask_create(ctx, P, [r[0] for r in runs], [r[1] for r in runs])
    enc_idx, plain_idx = ofed.mask_indices(P, runs)
    rs = np.random.default_rng(30 + limbs)
    w = rs.normal(0, 0.05, P).astype(np.float32)
    ct, pl = he.he_encrypt_masked(ctx, keys, mask, SEED + 5, 2, _dev(w))
    ct_h = _np(ct).astype(np.int64)
    for level in range(1, limbs + 1):
        cut = ct[:, :, :level].contiguous()
        out = _np(he.he_decrypt_merge_level(ctx, keys, mask, level, cut, pl))
        assert np.array_equal(out[plain_idx], w[plain_idx])
        for c in range(mask.n_ct):
            z = ofed.decode_ct_level(p, okeys, ct_h[c][:, :level], level)
            sel = enc_idx[c * n:(c + 1) * n]
            assert np.abs(out[sel].astype(np.float64) - z[:len(sel)].astype(np.float32).astype(np.float64)).max() <= 1e-6, (level, c)
        assert np.abs(out[enc_idx] - w[enc_idx]).max() < 16 * ofed.noise_sigma(p, [1.0])
    for bad in (0, limbs + 1):
        with pytest.raises(he.HeError):
            he.he_decrypt_merge_level(ctx, keys, mask, bad, torch.zeros((mask.n_ct, 2, bad, ctx.N), dtype=torch.int32, device="cuda"), pl)
    mask.close()


def _gpu_round(he, ctx, keys, mask, ws, alpha, seed):
    cts, plains = [], []
    for i, w in enumerate(ws):
        ct, pl = he.he_encrypt_masked(ctx, keys, mask, seed, i, w)
        cts.append(ct)
        plains.append(pl)
    ct_g, pl_g = he.he_aggregate(ctx, alpha, cts, plains)
    out = he.he_decrypt_merge(ctx, keys, mask, ct_g, pl_g)
    return cts, plains, ct_g, pl_g, out


MASK_CASES = {
    "full": lambda P, n: [(0, P)],
    "empty": lambda P, n: [],
    "ragged": lambda P, n: [(3, 1), (5, 1), (7, n + 9), (2 * n + 50, 2 * n), (P - 1, 1)],
    "multiple_of_n": lambda P, n: [(11, 2 * n)],
    "short": lambda P, n: [(P // 2, 5)],
}


@pytest.mark.parametrize("case", list(MASK_CASES))
@pytest.mark.parametrize("log2_n,limbs", [(10, 3), (12, 3), (13, 3)])
def test_round_small(he, log2_n, limbs, case):
    """Whole path on small vectors, every ciphertext checked: gather, encode (+-1), encrypt
    (bit-exact given the GPU's plaintext), aggregate (bit-exact), decrypt+decode+merge (1e-6)."""
    ctx, keys, p, okeys = _setup(he, log2_n, limbs)
    n = p.n_slots
    P = 5 * n + 123
    runs = MASK_CASES[case](P, n)
    mask = he.he_mask_create(ctx, P, [r[0] for r in runs], [r[1] for r in runs])
    enc_idx, plain_idx = ofed.mask_indices(P, runs)
    assert mask.P_enc == len(enc_idx) and mask.n_ct == ofed.n_ciphertexts(p, len(enc_idx))
    K = 3
    rs = np.random.default_rng(6)
    ws = [rs.normal(0, 0.05, P).astype(np.float32) for _ in range(K)]
    alpha = np.array([0.5, 0.3, 0.2])
    cts, plains, ct_g, pl_g, out = _gpu_round(he, ctx, keys, mask, [_dev(w) for w in ws], alpha, SEED)
    out = _np(out)
    o_cts = []
    for i in range(K):
        assert np.array_equal(_np(plains[i]), ws[i][plain_idx])
        ct_i = _np(cts[i]).astype(np.int64)
        row = []
        for c in range(mask.n_ct):
            z = ofed.pack_slots(p, ws[i], enc_idx, c)
            m_gpu = _np(he.he_debug_encode(ctx, _dev(z.astype(np.float32)[None])))[0].astype(np.int64)
            assert np.abs(m_gpu - oenc.encode_fft(z, log2_n, 30)).max() <= 1
            ref = osch.encrypt(p, okeys, m_gpu, SEED, i, c)
            assert np.array_equal(ct_i[c], ref), (i, c)
            row.append(ref)
        o_cts.append(row)
    ct_gn = _np(ct_g).astype(np.int64)
    expect = np.zeros(P, dtype=np.float32)
    expect[plain_idx] = ofed.plain_fedavg([w[plain_idx] for w in ws], alpha)
    for c in range(mask.n_ct):
        agg = osch.aggregate(p, [o_cts[i][c] for i in range(K)], alpha)
        assert np.array_equal(ct_gn[c], agg)
        z = ofed.decode_ct(p, okeys, agg)
        sel = enc_idx[c * n:(c + 1) * n]
        expect[sel] = z[:len(sel)].astype(np.float32)
    assert np.array_equal(out[plain_idx], expect[plain_idx])
    assert np.abs(out.astype(np.float64) - expect.astype(np.float64)).max() <= 1e-6
    # against exact FedAvg: inside the CKKS noise model
    ref = ofed.fedavg_float64(ws, alpha)
    if len(enc_idx):
        assert np.abs(out[enc_idx] - ref[enc_idx]).max() < 16 * ofed.noise_sigma(p, alpha)
    # determinism: the same call again gives the same bytes
    ct_again, _ = he.he_encrypt_masked(ctx, keys, mask, SEED, 0, _dev(ws[0]))
    assert torch.equal(ct_again, cts[0])


@pytest.mark.parametrize("log2_n,limbs,K", [(10, 2, 3), (13, 2, 5), (14, 3, 8), (10, 3, 70)])
def test_client_weighted_variant(he, log2_n, limbs, K):
    """Weighing on the client, the server only adds: every step against the oracle."""
    ctx, keys, p, okeys = _setup(he, log2_n, limbs)
    n = p.n_slots
    P = 2 * n + 777
    runs = [(5, n + 100), (n + 300, n // 2)]
    mask = he.he_mask_create(ctx, P, [r[0] for r in runs], [r[1] for r in runs])
    enc_idx, plain_idx = ofed.mask_indices(P, runs)
    rs = np.random.default_rng(8)
    ws = [rs.normal(0, 0.05, P).astype(np.float32) for _ in range(K)]
    counts = rs.integers(100, 1001, K)
    alpha = counts / counts.sum()
    cts, plains = [], []
    for i, w in enumerate(ws):
        ct, pl = he.he_encrypt_masked_weighted(ctx, keys, mask, SEED, i, alpha[i], _dev(w))
        cts.append(ct)
        plains.append(pl)
        assert np.array_equal(_np(pl), ofed.plain_weighted(w[plain_idx], alpha[i]))
    ct_g, pl_g = he.he_aggregate_sum(ctx, cts, plains)
    out = _np(he.he_decrypt_merge_level(ctx, keys, mask, limbs, ct_g, pl_g))
    assert np.array_equal(_np(pl_g), ofed.plain_sum([_np(x) for x in plains]))
    ct_gn = _np(ct_g).astype(np.int64)
    expect = np.zeros(P, dtype=np.float32)
    expect[plain_idx] = _np(pl_g)
    checked_clients = range(K) if K <= 8 else [0, K - 1]
    for c in range(mask.n_ct):
        for i in checked_clients:
            z = np.float64(alpha[i]) * ofed.pack_slots(p, ws[i], enc_idx, c)
            ref = osch.encrypt(p, okeys, oenc.encode_fft(z, log2_n, 30), SEED, i, c)
            ct_i = _np(cts[i][c]).astype(np.int64)
            # c1 does not involve the plaintext: bit-exact.  c0 differs from the oracle's by the encoder's
            # +-1 tolerance only, the same small integer in every limb.
            assert np.array_equal(ct_i[1], ref[1])
            d0 = None
            for j, q in enumerate(p.primes):
                dj = (ct_i[0, j] - ref[0, j]) % q
                dj = np.where(dj > q // 2, dj - q, dj)
                assert np.abs(dj).max() <= 1 and (dj != 0).mean() < 1e-3
                assert d0 is None or np.array_equal(dj, d0)
                d0 = dj
        agg = osch.sum_ciphertexts(p, [_np(cts[i][c]).astype(np.int64) for i in range(K)])
        assert np.array_equal(ct_gn[c], agg)
        zdec = ofed.decode_ct_level(p, okeys, agg, limbs)
        sel = enc_idx[c * n:(c + 1) * n]
        expect[sel] = zdec[:len(sel)].astype(np.float32)
    assert np.array_equal(out[plain_idx], expect[plain_idx])
    assert np.abs(out.astype(np.float64) - expect.astype(np.float64)).max() <= 1e-6
    ref = ofed.fedavg_float64(ws, alpha)
    assert np.abs(out[enc_idx] - ref[enc_idx]).max() < 16 * ofed.noise_sigma_client_weighted(p, K)


@pytest.mark.parametrize("log2_n,limbs", [(13, 8), (14, 2), (12, 5), (14, 6)])
def test_round_other_chain_lengths(he, log2_n, limbs):
    """Chain lengths other than the benchmark's (shortest, longest, and the long ones on both specialised rings):
    whole round, every ciphertext bit-exact, decoded values within 1e-6."""
    ctx, keys, p, okeys = _setup(he, log2_n, limbs)
    n = p.n_slots
    P = n + n // 2 + 5
    runs = [(2, n), (n + 10, n // 2 - 7)]
    mask = he.he_mask_create(ctx, P, [r[0] for r in runs], [r[1] for r in runs])
    enc_idx, plain_idx = ofed.mask_indices(P, runs)
    rs = np.random.default_rng(10 + limbs)
    K = 2
    ws = [rs.normal(0, 0.05, P).astype(np.float32) for _ in range(K)]
    alpha = np.array([0.625, 0.375])
    cts, plains, ct_g, pl_g, out = _gpu_round(he, ctx, keys, mask, [_dev(w) for w in ws], alpha, SEED)
    out = _np(out)
    expect = np.zeros(P, dtype=np.float32)
    expect[plain_idx] = ofed.plain_fedavg([w[plain_idx] for w in ws], alpha)
    for c in range(mask.n_ct):
        refs = []
        for i in range(K):
            z = ofed.pack_slots(p, ws[i], enc_idx, c)
            m_gpu = _np(he.he_debug_encode(ctx, _dev(z.astype(np.float32)[None])))[0].astype(np.int64)
            ref = osch.encrypt(p, okeys, m_gpu, SEED, i, c)
            assert np.array_equal(_np(cts[i][c]).astype(np.int64), ref), (i, c)
            refs.append(ref)
        agg = osch.aggregate(p, refs, alpha)
        assert np.array_equal(_np(ct_g[c]).astype(np.int64), agg)
        sel = enc_idx[c * n:(c + 1) * n]
        expect[sel] = ofed.decode_ct(p, okeys, agg)[:len(sel)].astype(np.float32)
    assert np.array_equal(out[plain_idx], expect[plain_idx])
    assert np.abs(out.astype(np.float64) - expect.astype(np.float64)).max() <= 1e-6


@pytest.mark.parametrize("log2_n,limbs,seed", [(10, 3, 0), (11, 3, 3), (13, 3, 1), (14, 4, 2)])
def test_round_random_fragmented_masks(he, log2_n, limbs, seed):
    """Masks made of hundreds of short random runs (many of length 1, many ciphertexts that straddle dozens of runs):
    gather, compaction, scatter and merge against the oracle over the whole vector."""
    ctx, keys, p, okeys = _setup(he, log2_n, limbs)
    n = p.n_slots
    rs = np.random.default_rng(100 + seed)
    P = 3 * n + int(rs.integers(1, n))
    cuts = np.sort(rs.choice(np.arange(1, P), size=min(P // 3, 1200), replace=False))
    bounds = np.concatenate([[0], cuts, [P]])
    runs = [(int(bounds[i]), int(bounds[i + 1] - bounds[i])) for i in range(int(rs.integers(0, 2)), len(bounds) - 1, 2)]
    mask = he.he_mask_create(ctx, P, [r[0] for r in runs], [r[1] for r in runs])
    enc_idx, plain_idx = ofed.mask_indices(P, runs)
    K = 2
    ws = [rs.normal(0, 0.05, P).astype(np.float32) for _ in range(K)]
    alpha = np.array([0.3, 0.7])
    cts, plains, ct_g, pl_g, out = _gpu_round(he, ctx, keys, mask, [_dev(w) for w in ws], alpha, SEED)
    for i in range(K):
        assert np.array_equal(_np(plains[i]), ws[i][plain_idx])
    expect = ofed.secure_round(p, okeys, ws, alpha, runs, SEED)
    out = _np(out)
    assert np.array_equal(out[plain_idx], expect[plain_idx])
    # the encoder's +-1 tolerance moves a decoded slot by about 2^-30 * sqrt(N): far inside 1e-6
    assert np.abs(out.astype(np.float64) - expect.astype(np.float64)).max() <= 1e-6


def test_mask_from_bytes_and_errors(he):
    ctx, keys, p, _ = _setup(he, 10, 3)
    P = 5000
    rs = np.random.default_rng(7)
    m = (rs.random(P) < 0.3).astype(np.uint8)
    mask = he.he_mask_from_bytes(ctx, _dev(m))
    assert mask.P == P and mask.P_enc == int(m.sum())
    w = rs.normal(0, 0.05, P).astype(np.float32)
    _, plain = he.he_encrypt_masked(ctx, keys, mask, SEED, 0, _dev(w))
    assert np.array_equal(_np(plain), w[m == 0])
    for starts, lens in ([[10, 5], [3, 3]], [[0, 4], [5, 3]], [[0], [P + 1]], [[3], [0]]):
        with pytest.raises(he.HeError):
            he.he_mask_create(ctx, P, starts, lens)
    # ciphertext buffers must be 16-byte aligned
    buf = torch.empty(mask.n_ct * 2 * ctx.L * ctx.N + 1, dtype=torch.int32, device="cuda")
    with pytest.raises(he.HeError):
        he.he_encrypt_masked(ctx, keys, mask, SEED, 0, _dev(w), buf[1:])
    with pytest.raises(he.HeError):
        he.Context(16, 3)
    with pytest.raises(he.HeError):
        he.Context(10, 1)


def test_input_range_check(he):
    """he_debug_count_out_of_range counts exactly the entries the encoder cannot carry."""
    ctx, _, p, _ = _setup(he, 10, 3)
    rs = np.random.default_rng(11)
    w = rs.normal(0, 0.05, 300_001).astype(np.float32)
    assert he.he_debug_count_out_of_range(ctx, _dev(w)) == 0
    bad = {5: np.nan, 17: np.inf, 99: -np.inf, 1000: 2.0, 2000: -2.0, 300_000: 1e30}
    fine = {7: np.float32(2.0) - np.float32(2.0 ** -22), 8: -(np.float32(2.0) - np.float32(2.0 ** -22)), 9: 0.0, 10: -0.0}
    for k, v in {**bad, **fine}.items():
        w[k] = v
    ref = int(np.sum(~(np.abs(w.astype(np.float64)) * 2.0 ** 30 < 2.0 ** 31 - 32)))
    assert ref == len(bad)
    assert he.he_debug_count_out_of_range(ctx, _dev(w)) == ref
    assert he.he_debug_count_out_of_range(ctx, torch.empty(0, dtype=torch.float32, device="cuda")) == 0


@pytest.mark.parametrize("log2_n,limbs", [(10, 3), (13, 3)])
def test_degenerate_sizes(he, log2_n, limbs):
    """The smallest inputs: an empty model, one parameter (encrypted, or left plain), one parameter more than a ciphertext."""
    ctx, keys, p, okeys = _setup(he, log2_n, limbs)
    n = p.n_slots
    alpha = np.array([0.25, 0.75])
    for P, runs in ((0, []), (1, [(0, 1)]), (1, []), (n + 1, [(0, n + 1)]), (2, [(1, 1)])):
        mask = he.he_mask_create(ctx, P, [r[0] for r in runs], [r[1] for r in runs])
        enc_idx, plain_idx = ofed.mask_indices(P, runs)
        assert mask.P == P and mask.P_enc == len(enc_idx) and mask.n_ct == ofed.n_ciphertexts(p, len(enc_idx))
        rs = np.random.default_rng(P + len(runs))
        ws = [rs.normal(0, 0.05, P).astype(np.float32) for _ in range(2)]
        cts, plains, ct_g, pl_g, out = _gpu_round(he, ctx, keys, mask, [_dev(w) for w in ws], alpha, SEED)
        out = _np(out)
        assert out.shape == (P,)
        expect = ofed.secure_round(p, okeys, ws, alpha, runs, SEED)
        # the GPU's encoder may differ from the oracle's by one unit in a coefficient: 2^-30 in a slot at most n times over
        assert np.array_equal(out[plain_idx], expect[plain_idx])
        if len(enc_idx):
            assert np.abs(out[enc_idx].astype(np.float64) - expect[enc_idx].astype(np.float64)).max() <= 1e-6
        mask.close()


def test_three_training_rounds(he):
    """Algorithm 1's loop, T = 3 rounds with one context, key pair and mask: decrypt + merge, a stand-in for local
    training (every client adds its own small update), encrypt, aggregate.  Each round is checked against the oracle's
    round on the same inputs, and the final model against the float64 FedAvg recursion under the noise model (fresh
    noise every round: the per-round seeds differ, so three independent errors add up)."""
    ctx, keys, p, okeys = _setup(he, 13, 3)
    n = p.n_slots
    P = 3 * n + 500
    runs = [(100, n + 50), (2 * n, n // 2)]
    mask = he.he_mask_create(ctx, P, [r[0] for r in runs], [r[1] for r in runs])
    enc_idx, _ = ofed.mask_indices(P, runs)
    K = 3
    alpha = np.array([0.2, 0.3, 0.5])
    rs = np.random.default_rng(12)
    glob_gpu = rs.normal(0, 0.05, P).astype(np.float32)
    glob_ref = glob_gpu.astype(np.float64)
    for t in range(3):
        updates = [rs.normal(0, 0.01, P).astype(np.float32) for _ in range(K)]
        ws = [(glob_gpu + u).astype(np.float32) for u in updates]                       # "Train"
        glob_ref = sum(a * (glob_ref + u.astype(np.float64)) for a, u in zip(alpha, updates))
        seed = SEED + 1000 * t
        _, _, _, _, out = _gpu_round(he, ctx, keys, mask, [_dev(w) for w in ws], alpha, seed)
        out = _np(out)
        expect = ofed.secure_round(p, okeys, ws, alpha, runs, seed)
        assert np.abs(out.astype(np.float64) - expect.astype(np.float64)).max() <= 1e-6, t
        glob_gpu = out
    sigma = ofed.noise_sigma(p, alpha)
    err = glob_gpu.astype(np.float64) - glob_ref
    plain = np.setdiff1d(np.arange(P), enc_idx)
    assert np.abs(err[plain]).max() < 3e-7                                               # float32 rounding of the plain part, three times
    assert np.abs(err[enc_idx]).max() < 16 * sigma * np.sqrt(3)
    assert 0.6 * sigma < err[enc_idx].std() < 1.4 * sigma * np.sqrt(3)
    mask.close()


def test_noncanonical_residue_count(he):
    """he_debug_count_noncanonical counts exactly the words that are not below their limb's prime, at both levels."""
    ctx, keys, p, _ = _setup(he, 10, 3)
    rs = np.random.default_rng(13)
    for level in (3, 2):
        ct = np.stack([rs.integers(0, q, (5, 2, p.N)) for q in p.primes[:level]], axis=2).astype(np.int64)
        assert he.he_debug_count_noncanonical(ctx, _dev(ct, torch.int32), level) == 0
        bad = ct.copy()
        bad[0, 0, 0, 0] = p.primes[0]                    # q itself
        bad[4, 1, level - 1, p.N - 1] = 2 ** 32 - 1      # the largest word
        bad[2, 1, 1, 7] = p.primes[1] + 5
        bad[3, 0, 1, 9] = p.primes[1] - 1                # still canonical
        as_i32 = torch.from_numpy(bad.astype(np.uint32).view(np.int32)).cuda()
        assert he.he_debug_count_noncanonical(ctx, as_i32, level) == 3
    # what the library itself produces is canonical
    mask = he.he_mask_create(ctx, 3 * p.n_slots, [0], [3 * p.n_slots])
    ct, _ = he.he_encrypt_masked(ctx, keys, mask, SEED, 0, _dev(rs.normal(0, 0.05, 3 * p.n_slots).astype(np.float32)))
    assert he.he_debug_count_noncanonical(ctx, ct, 3) == 0
    assert he.he_debug_count_noncanonical(ctx, torch.empty((0, 2, 3, p.N), dtype=torch.int32, device="cuda"), 3) == 0
