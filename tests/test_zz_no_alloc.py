"""he_encrypt_masked_static (the entry point that allocates nothing) against he_encrypt_masked, through the C ABI:
identical ciphertext and remainder bytes on two calls in a row, the second with a smaller input; sizes beyond the static
scratch are refused; free device memory does not move across the calls."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

SEED = 0xA110C


@pytest.fixture(scope="module")
def he():
    from paper_2303_10837_amd import binding
    binding.load()
    torch.cuda.set_device(0)
    return binding


def _mask(he, ctx, P, runs):
    return he.he_mask_create(ctx, P, [r[0] for r in runs], [r[1] for r in runs])


@pytest.mark.parametrize("log2_n,limbs", [(13, 3), (14, 4), (10, 3)])
def test_static_scratch_entry_point_matches_the_allocating_one(he, log2_n, limbs):
    rs = np.random.default_rng(log2_n)
    ref_ctx = he.Context(log2_n, limbs)             # grows its own scratch on demand
    ref_keys = he.he_keygen(ref_ctx, SEED)
    ctx = he.Context(log2_n, limbs)                 # only ever used through the static entry point
    keys = he.he_keygen(ctx, SEED)
    n = ctx.n_slots
    big = (7 * n + 1234 + 3 * n, [(5, 3 * n + 17), (4 * n, 2 * n), (7 * n + 100, n + 500)])      # 7 ciphertexts, ragged tail
    small = (2 * n + 99, [(n // 2, n + 3)])                                                      # 2 ciphertexts
    frag = (6 * n + 5, [(i * 37 + 2, 11) for i in range((6 * n) // 37)])                         # runs of 11 every 37: the fragmented-mask kernels
    torch.cuda.synchronize()
    for P, runs in (big, frag, small):
        w = torch.from_numpy(rs.normal(0, 0.05, P).astype(np.float32)).cuda()
        m_ref, m = _mask(he, ref_ctx, P, runs), _mask(he, ctx, P, runs)
        ct_ref, pl_ref = he.he_encrypt_masked(ref_ctx, ref_keys, m_ref, SEED + 1, 4, w)
        ct = torch.full((m.n_ct, 2, ctx.L, ctx.N), -1, dtype=torch.int32, device="cuda")
        pl = torch.full((m.n_plain,), float("nan"), dtype=torch.float32, device="cuda")
        torch.cuda.synchronize()
        free_before = torch.cuda.mem_get_info()[0]
        he.he_encrypt_masked_static(ctx, keys, m, SEED + 1, 4, w, ct, pl)
        torch.cuda.synchronize()
        assert torch.cuda.mem_get_info()[0] == free_before          # nothing allocated, nothing freed
        assert m.n_ct == m_ref.n_ct and m.n_ct >= 2
        assert torch.equal(ct, ct_ref) and torch.equal(pl, pl_ref)   # integers and copied floats: bit for bit
        m_ref.close()
        m.close()
    # beyond the static scratch: refused with a message, nothing written
    per_ct = 7 * ctx.N
    too_many = he.HE_STATIC_SCRATCH_BYTES // per_ct + 1
    P = too_many * n
    m = _mask(he, ctx, P, [(0, P)])
    assert m.n_ct == too_many
    w = torch.zeros(P, dtype=torch.float32, device="cuda")
    ct = torch.zeros((m.n_ct, 2, ctx.L, ctx.N), dtype=torch.int32, device="cuda")
    with pytest.raises(he.HeError, match="static scratch"):
        he.he_encrypt_masked_static(ctx, keys, m, SEED, 0, w, ct, torch.empty(0, dtype=torch.float32, device="cuda"))
    assert int(ct.abs().max()) == 0
    # exactly at the limit it still runs (same bytes as the allocating entry point on the last ciphertext)
    P = (too_many - 1) * n
    m = _mask(he, ctx, P, [(0, P)])
    m_ref = _mask(he, ref_ctx, P, [(0, P)])
    w = torch.from_numpy(rs.normal(0, 0.05, P).astype(np.float32)).cuda()
    ct = torch.empty((m.n_ct, 2, ctx.L, ctx.N), dtype=torch.int32, device="cuda")
    he.he_encrypt_masked_static(ctx, keys, m, SEED + 2, 1, w, ct, torch.empty(0, dtype=torch.float32, device="cuda"))
    ct_ref, _ = he.he_encrypt_masked(ref_ctx, ref_keys, m_ref, SEED + 2, 1, w)
    assert torch.equal(ct, ct_ref)
    for x in (m, m_ref, keys, ref_keys, ctx, ref_ctx):
        x.close()
