"""A whole round captured in a HIP graph replays to the bytes of the eager round.

The library's calls only enqueue work on the given stream, allocate nothing once the context's scratch has grown to the workload's size in a first eager
call, and clear memory with kernels, not memset nodes: so a round can be captured and replayed.  Every replay is
checked, with eager work and synchronisations of the same context in between.
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("log2_n,limbs", [(10, 3), (13, 3)])
def test_graph_replay_matches_eager(log2_n, limbs):
    from paper_2303_10837_amd import binding as he
    he.load()
    torch.cuda.set_device(0)
    ctx = he.Context(log2_n, limbs)
    keys = he.he_keygen(ctx, 99)
    n = ctx.n_slots
    P = 6 * n + 321
    runs = [(5, 2 * n + 7), (3 * n, n), (5 * n + 11, 300)]            # selective: a plaintext remainder is compacted and scattered too
    mask = he.he_mask_create(ctx, P, [r[0] for r in runs], [r[1] for r in runs])
    K = 3
    rs = np.random.default_rng(0)
    ws = [torch.from_numpy(rs.normal(0, 0.05, P).astype(np.float32)).cuda() for _ in range(K)]
    alpha = np.array([0.2, 0.5, 0.3])
    cts = [torch.empty((mask.n_ct, 2, ctx.L, ctx.N), dtype=torch.int32, device="cuda") for _ in range(K)]
    pls = [torch.empty((mask.n_plain,), dtype=torch.float32, device="cuda") for _ in range(K)]
    ct_g = torch.empty((mask.n_ct, 2, ctx.L - 1, ctx.N), dtype=torch.int32, device="cuda")
    pl_g = torch.empty((mask.n_plain,), dtype=torch.float32, device="cuda")
    out = torch.empty((P,), dtype=torch.float32, device="cuda")

    def round_():
        for i in range(K):
            he.he_encrypt_masked(ctx, keys, mask, 7, i, ws[i], cts[i], pls[i])
        he.he_aggregate(ctx, alpha, cts, pls, ct_g, pl_g)
        he.he_decrypt_merge(ctx, keys, mask, ct_g, pl_g, out)

    round_()                                                           # eager: also grows the scratch to its size
    torch.cuda.synchronize()
    ref = [t.clone() for t in (*cts, *pls, ct_g, pl_g, out)]
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        round_()
    for replay in range(3):
        for t in (*cts, *pls, ct_g, pl_g, out):
            t.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for got, want in zip((*cts, *pls, ct_g, pl_g, out), ref):
            assert torch.equal(got, want), f"replay {replay} differs from the eager round"
        # eager work of the same context between the replays (other inputs, so stale results would show)
        he.he_encrypt_masked(ctx, keys, mask, 8, 0, ws[1], cts[0], pls[0])
        torch.cuda.synchronize()
    keys.close()
    mask.close()
    ctx.close()
