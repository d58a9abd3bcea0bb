"""GPU parity of the encryption-mask agreement: Select(global privacy map, p) and the run
extraction, bit for bit against the oracle, and the whole flow of Algorithm 1's first phase
(clients encrypt sensitivity maps, the server aggregates, the map is decrypted, the mask selected)."""
import numpy as np
import pytest
import torch

from oracle import encoder as oenc
from oracle import fedavg as ofed
from oracle import scheme as osch
from oracle import select as osel
from oracle.params import Params

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def he():
    from paper_2303_10837_amd import binding
    binding.load()
    torch.cuda.set_device(0)
    return binding


@pytest.fixture(scope="module")
def ctx(he):
    return he.Context(10, 3)


def _runs(he, mask):
    starts, lens = he.he_mask_runs(mask)
    return list(zip(starts, lens))


def _sens_cases():
    rs = np.random.default_rng(5)
    P = 3 * 2048 + 1234                                      # several chunks and a ragged tail
    yield "gaussian", np.abs(rs.normal(0, 1, P)).astype(np.float32)
    yield "signed", rs.normal(0, 1, P).astype(np.float32)
    yield "few_levels", rs.integers(0, 5, P).astype(np.float32)          # heavy ties: the threshold is shared
    z = np.abs(rs.normal(0, 1, P)).astype(np.float32)
    z[rs.random(P) < 0.6] = 0.0
    z[rs.integers(0, P, 50)] = -0.0
    yield "mostly_zero", z
    blocks = np.repeat(rs.random(P // 64 + 1).astype(np.float32), 64)[:P] + rs.random(P).astype(np.float32) * 1e-3
    yield "layerwise", blocks
    yield "constant", np.full(P, 0.25, dtype=np.float32)
    yield "tiny", np.array([3.0, 1.0, 2.0], dtype=np.float32)
    yield "single", np.array([1.0], dtype=np.float32)
    yield "denormal_and_large", np.concatenate([np.float32(1e-42) * rs.integers(0, 9, 3000), np.float32(1e30) * rs.random(3000)]).astype(np.float32)


@pytest.mark.parametrize("name,sens", list(_sens_cases()))
def test_select_top_matches_oracle(he, ctx, name, sens):
    d = torch.from_numpy(sens).cuda()
    for ratio in (0.0, 0.001, 0.1, 0.3, 0.5, 0.77, 1.0):
        mask = he.he_mask_select_top(ctx, d, ratio)
        want = osel.select_top(sens, ratio)
        assert mask.P == len(sens) and mask.P_enc == int(want.sum()) == osel.select_count(len(sens), ratio)
        assert _runs(he, mask) == osel.runs_of(want), (name, ratio)
        mask.close()


def test_mask_from_bytes_run_extraction(he, ctx):
    rs = np.random.default_rng(6)
    for P, density in ((1, 1.0), (5000, 0.3), (2048, 0.5), (2049, 0.99), (4 * 2048, 0.01), (3 * 2048 + 7, 0.0)):
        m = (rs.random(P) < density).astype(np.uint8) * rs.integers(1, 255, P).astype(np.uint8)   # any non-zero byte counts
        mask = he.he_mask_from_bytes(ctx, torch.from_numpy(m).cuda())
        assert _runs(he, mask) == osel.runs_of(m != 0)
        mask.close()
    # boundaries: runs that start / end exactly at chunk edges
    m = np.zeros(3 * 2048, dtype=np.uint8)
    m[0:8] = 1; m[2040:2048] = 1; m[2048:2056] = 1; m[4095] = 1; m[4096] = 1; m[-1] = 1
    mask = he.he_mask_from_bytes(ctx, torch.from_numpy(m).cuda())
    assert _runs(he, mask) == osel.runs_of(m != 0) == [(0, 8), (2040, 16), (4095, 2), (6143, 1)]


def test_select_extreme_counts(he, ctx):
    """k = 1 and k = P - 1 (one entry selected, one entry left out), with the extreme value at either end, in the
    middle and tied with another entry."""
    rs = np.random.default_rng(12)
    P = 2 * 2048 + 333
    base = rs.random(P).astype(np.float32)
    for where in (0, P - 1, P // 2):
        for sign, ratio in ((+1.0, 1.0 / P), (-1.0, (P - 1.0) / P)):
            sens = base.copy()
            sens[where] = sign * 5.0                          # the single largest / smallest entry
            mask = he.he_mask_select_top(ctx, torch.from_numpy(sens).cuda(), ratio)
            want = osel.select_top(sens, ratio)
            assert int(want.sum()) == (1 if sign > 0 else P - 1) and want[where] == (sign > 0)
            assert _runs(he, mask) == osel.runs_of(want)
            mask.close()
    sens = base.copy()
    sens[[5, 4000]] = 7.0                                     # two entries tied for the top: the lower index wins
    mask = he.he_mask_select_top(ctx, torch.from_numpy(sens).cuda(), 1.0 / P)
    assert _runs(he, mask) == [(5, 1)]
    mask.close()


def test_unaligned_vectors(he, ctx):
    """Vectors that start at an odd element of an allocation (4-byte and 1-byte aligned only): the kernels' wide
    loads and stores do not apply, the results are the same."""
    rs = np.random.default_rng(8)
    P = 5 * 2048 + 77
    sens = np.abs(rs.normal(0, 1, P + 3)).astype(np.float32)
    sens[rs.integers(0, P, 400)] = sens[17]                      # ties at some values
    d = torch.from_numpy(sens).cuda()
    for off in (1, 2, 3):
        view = d[off:off + P]
        assert view.data_ptr() % 16 == 4 * off
        for ratio in (0.1, 0.5):
            mask = he.he_mask_select_top(ctx, view, ratio)
            assert _runs(he, mask) == osel.runs_of(osel.select_top(sens[off:off + P], ratio))
            mask.close()
    m = (rs.random(P + 7) < 0.4).astype(np.uint8)
    dm = torch.from_numpy(m).cuda()
    for off in (1, 3, 4, 7):
        mask = he.he_mask_from_bytes(ctx, dm[off:off + P])
        assert _runs(he, mask) == osel.runs_of(m[off:off + P] != 0)
        mask.close()


def test_select_large_vector_properties(he, ctx):
    """25.6M entries (the ResNet-50-sized workload), layer-structured sensitivities: the selection has exactly k
    entries, every selected value is >= every unselected one, and sampled windows match the oracle's definition."""
    P, ratio = 25_600_000, 0.1
    g = torch.Generator(device="cuda").manual_seed(7)
    layer = torch.rand(P // 4096 + 1, generator=g, device="cuda").repeat_interleave(4096)[:P]
    sens = (layer + 0.05 * torch.rand(P, generator=g, device="cuda")).float()
    mask = he.he_mask_select_top(ctx, sens, ratio)
    k = osel.select_count(P, ratio)
    assert mask.P_enc == k
    starts, lens = he.he_mask_runs(mask)
    sel = torch.zeros(P + 1, dtype=torch.int32, device="cuda")
    st = torch.tensor(starts, device="cuda", dtype=torch.int64)
    ln = torch.tensor(lens, device="cuda", dtype=torch.int64)
    sel.index_add_(0, st, torch.ones_like(st, dtype=torch.int32))
    sel.index_add_(0, st + ln, -torch.ones_like(st, dtype=torch.int32))
    sel = sel.cumsum(0)[:P].bool()
    assert int(sel.sum()) == k
    lo_sel, hi_unsel = float(sens[sel].min()), float(sens[~sel].max())
    assert lo_sel >= hi_unsel
    if lo_sel == hi_unsel:   # ties at the threshold: lower indices first
        eq = (sens == lo_sel).nonzero().flatten()
        taken = sel[eq]
        assert bool((taken[:-1] >= taken[1:]).all())


def test_mask_agreement_flow(he):
    """Clients encrypt sensitivity maps (everything encrypted), the server forms the global privacy map
    homomorphically, it is decrypted and the top-p mask selected; that mask then drives a selective round."""
    log2_n, L, K, seed = 10, 3, 4, 99
    ctx = he.Context(log2_n, L)
    keys = he.he_keygen(ctx, seed)
    p = Params(log2_n, L)
    n = p.n_slots
    P = 6 * n + 300
    rs = np.random.default_rng(9)
    layer_scale = np.repeat(rs.random(P // 128 + 1), 128)[:P]
    sens = [np.abs(rs.normal(0, 1, P) * 0.02 + layer_scale * (0.5 + 0.1 * i)).astype(np.float32) for i in range(K)]
    counts = rs.integers(100, 1001, K)
    alpha = counts / counts.sum()
    full = he.he_mask_create(ctx, P, [0], [P])
    cts = [he.he_encrypt_masked(ctx, keys, full, seed, i, torch.from_numpy(s).cuda())[0] for i, s in enumerate(sens)]
    ct_g, _ = he.he_aggregate(ctx, alpha, cts, [None] * K)
    gmap = he.he_decrypt_merge(ctx, keys, full, ct_g, None)
    # the decrypted map is the weighted mean of the sensitivity maps up to the CKKS noise
    ref = ofed.fedavg_float64(sens, alpha)
    assert np.abs(gmap.cpu().numpy() - ref).max() < 16 * ofed.noise_sigma(p, alpha)
    ratio = 0.3
    mask = he.he_mask_select_top(ctx, gmap, ratio)
    want = osel.select_top(gmap.cpu().numpy(), ratio)
    assert _runs(he, mask) == osel.runs_of(want)
    # the noise (1e-5) is far below the layer structure (0.1 and more): the selection agrees with the exact map's
    exact = osel.select_top(ref.astype(np.float32), ratio)
    assert (want != exact).mean() < 2e-3
    # and the mask is usable as it is
    w = rs.normal(0, 0.05, P).astype(np.float32)
    ct, plain = he.he_encrypt_masked(ctx, keys, mask, seed, 0, torch.from_numpy(w).cuda())
    assert ct.shape[0] == mask.n_ct and np.array_equal(plain.cpu().numpy(), w[~want])


def test_fragmented_mask_on_unaligned_model_vectors(he):
    """Compaction and merge of the remainder under a fragmented mask when the model vector and the output start at an odd
    element of their allocations (the 16-byte accesses of the parameter-ordered kernels do not apply) and P is ragged."""
    ctx = he.Context(11, 2)
    keys = he.he_keygen(ctx, 3)
    rs = np.random.default_rng(14)
    for P in (4096 * 3 + 1, 4096 * 2, 70_001):
        m = rs.random(P) < 0.3
        mask = he.he_mask_from_bytes(ctx, torch.from_numpy(m.astype(np.uint8)).cuda())
        full = torch.from_numpy(rs.normal(0, 0.02, P + 3).astype(np.float32)).cuda()
        for off in (0, 1, 3):
            w = full[off:off + P]
            ct, pl = he.he_encrypt_masked(ctx, keys, mask, 9, 0, w)
            assert torch.equal(pl, w[torch.from_numpy(~m).cuda()])
            ct_g, pl_g = he.he_aggregate(ctx, [1.0], [ct], [pl])
            out_full = torch.full((P + 3,), float("nan"), device="cuda")
            out = he.he_decrypt_merge(ctx, keys, mask, ct_g, pl_g, out_full[off:off + P])
            assert torch.equal(out[torch.from_numpy(~m).cuda()], pl)
            assert float((out - w).abs().max()) < 1e-3                                   # masked entries: CKKS noise only
            untouched = torch.ones(P + 3, dtype=torch.bool)
            untouched[off:off + P] = False
            assert bool(torch.isnan(out_full.cpu()[untouched]).all())                    # nothing written outside the vector
        mask.close()


def test_round_under_a_per_parameter_selection(he):
    """A whole round under the mask a top-p selection over per-parameter sensitivities gives: runs of one or two
    parameters (about 180 k of them here), so that a ciphertext's slots and a chunk of the remainder span thousands of
    runs.  Compaction and merge are checked over the whole vector, sampled ciphertexts through every stage."""
    log2_n, L, K, seed = 13, 3, 3, 41
    ctx = he.Context(log2_n, L)
    keys = he.he_keygen(ctx, seed)
    p = Params(log2_n, L)
    okeys = osch.keygen(p, seed)
    n, P, ratio = p.n_slots, 2_000_003, 0.1
    rs = np.random.default_rng(13)
    sens = rs.random(P).astype(np.float32)
    mask = he.he_mask_select_top(ctx, torch.from_numpy(sens).cuda(), ratio)
    want = osel.select_top(sens, ratio)
    starts, lens = he.he_mask_runs(mask)
    assert len(starts) > 150_000 and list(zip(starts, lens)) == osel.runs_of(want)
    enc_idx, plain_idx = np.nonzero(want)[0], np.nonzero(~want)[0]
    assert mask.P_enc == len(enc_idx) and mask.n_ct == -(-len(enc_idx) // n)
    ws = [rs.normal(0, 0.02, P).astype(np.float32) for _ in range(K)]
    alpha = np.array([0.2, 0.5, 0.3])
    cts, pls = [], []
    for i in range(K):
        ct, pl = he.he_encrypt_masked(ctx, keys, mask, seed + 1, i, torch.from_numpy(ws[i]).cuda())
        assert np.array_equal(pl.cpu().numpy(), ws[i][plain_idx])                 # compaction, whole vector
        cts.append(ct); pls.append(pl)
    ct_g, pl_g = he.he_aggregate(ctx, alpha, cts, pls)
    out = he.he_decrypt_merge(ctx, keys, mask, ct_g, pl_g).cpu().numpy()
    assert np.array_equal(pl_g.cpu().numpy(), ofed.plain_fedavg([w[plain_idx] for w in ws], alpha))
    assert np.array_equal(out[plain_idx], pl_g.cpu().numpy())                      # scatter, whole vector
    for c in (0, mask.n_ct // 2, mask.n_ct - 1):                                   # the last one is ragged
        idx = enc_idx[c * n:(c + 1) * n]
        ct_c = []
        for i in range(K):
            z = np.zeros(n, dtype=np.float32)
            z[:len(idx)] = ws[i][idx]
            m = oenc.encode_fft(z.astype(np.float64), log2_n, 30)
            m_gpu = he.he_debug_encode(ctx, torch.from_numpy(z[None]).cuda())[0].cpu().numpy().astype(np.int64)
            assert np.abs(m_gpu - m).max() <= 1
            ref = osch.encrypt(p, okeys, m_gpu, seed + 1, i, c)
            assert np.array_equal(cts[i][c].cpu().numpy().astype(np.int64), ref), (i, c)   # the gather fed the right slots
            ct_c.append(ref)
        agg = osch.aggregate(p, ct_c, alpha)
        assert np.array_equal(ct_g[c].cpu().numpy().astype(np.int64), agg)
        zdec = ofed.decode_ct(p, okeys, agg)
        assert np.abs(out[idx].astype(np.float64) - zdec[:len(idx)].astype(np.float32).astype(np.float64)).max() <= 1e-6
    ref = ofed.fedavg_float64(ws, alpha)
    assert np.abs(out[enc_idx] - ref[enc_idx]).max() < 16 * ofed.noise_sigma(p, alpha)
