"""Pins for mask gather/scatter, packing and plain FedAvg (oracle side)."""
from fractions import Fraction

import numpy as np

from oracle import fedavg
from oracle.params import Params
from paper_2303_10837_amd import synth_inputs as si


def test_mask_partition_and_packing():
    p = Params(4, 3)                      # n = 8 slots
    P = 100
    w = np.arange(P, dtype=np.float32) + 0.5
    cases = [
        [(0, P)],                         # full mask
        [],                               # empty mask
        [(3, 1), (5, 1), (7, 9), (50, 8), (99, 1)],      # runs of length 1, straddling ciphertexts
        [(0, 16)],                        # P_enc multiple of n
        [(1, 17)],
    ]
    for runs in cases:
        enc_idx, plain_idx = fedavg.mask_indices(P, runs)
        assert len(enc_idx) == sum(l for _, l in runs)
        assert sorted(np.concatenate([enc_idx, plain_idx]).tolist()) == list(range(P))
        n_ct = fedavg.n_ciphertexts(p, len(enc_idx))
        assert n_ct == (len(enc_idx) + 7) // 8
        packed = np.concatenate([fedavg.pack_slots(p, w, enc_idx, c) for c in range(n_ct)]) if n_ct else np.zeros(0)
        assert np.array_equal(packed[:len(enc_idx)], w[enc_idx]) and np.all(packed[len(enc_idx):] == 0)
        back = np.full(P, -1.0, dtype=np.float32)
        back[enc_idx] = packed[:len(enc_idx)]
        back[plain_idx] = w[plain_idx]
        assert np.array_equal(back, w)


def test_plain_fedavg_against_exact_rationals():
    rs = np.random.default_rng(0)
    K, P = 5, 300
    ws = [rs.normal(0, 0.02, P).astype(np.float32) for _ in range(K)]
    counts = rs.integers(100, 1001, K)
    alpha = counts / counts.sum()
    out = fedavg.plain_fedavg(ws, alpha)
    assert out.dtype == np.float32
    for t in range(P):
        exact = sum(Fraction(float(a)) * Fraction(float(w[t])) for a, w in zip(alpha, ws))
        assert abs(Fraction(float(out[t])) - exact) <= Fraction(float(np.spacing(np.float32(abs(out[t])))))
    # special cases with exact answers
    assert np.array_equal(fedavg.plain_fedavg([ws[0]], [1.0]), ws[0])
    half = fedavg.plain_fedavg([ws[0], ws[1]], [0.5, 0.5])
    assert np.array_equal(half, ((ws[0].astype(np.float64) + ws[1].astype(np.float64)) / 2).astype(np.float32))


def test_synthetic_workload_recipes():
    for name, w in si.WORKLOADS.items():
        starts, lens = si.mask_runs(w)
        assert np.all(starts[1:] > starts[:-1] + lens[:-1]) if len(starts) > 1 else True
        assert int(starts[-1] + lens[-1]) <= w.n_params
        assert int(lens.sum()) == int(round(w.enc_ratio * w.n_params))
        a = si.client_alphas(w)
        assert a.shape == (w.n_clients,) and abs(a.sum() - 1) < 1e-12 and a.min() > 0
    w = si.scaled(si.WORKLOADS["bert_sel10"], 3_000_000)
    x = si.client_params_numpy(w, 1)
    assert x.dtype == np.float32 and x.shape == (3_000_000,) and 0.01 < x.std() < 0.05
    assert np.array_equal(x, si.client_params_numpy(w, 1)) and not np.array_equal(x, si.client_params_numpy(w, 2))
    x = si.client_params_numpy(si.WORKLOADS["tiny_full"], 0)
    assert abs(x.std() - 0.05) < 0.002


def test_run_list_lookup_matches_enumeration():
    rs = np.random.default_rng(3)
    P = 5000
    for trial in range(5):
        cuts = np.sort(rs.choice(np.arange(1, P), size=20, replace=False))
        bounds = np.concatenate([[0], cuts, [P]])
        runs = [(int(bounds[i]), int(bounds[i + 1] - bounds[i])) for i in range(trial % 2, len(bounds) - 1, 2)]
        starts, lens = [r[0] for r in runs], [r[1] for r in runs]
        enc_idx, plain_idx = fedavg.mask_indices(P, runs)
        t = np.arange(len(enc_idx))
        assert np.array_equal(fedavg.packed_to_param(starts, lens, t), enc_idx)
        cs, cl = fedavg.complement_runs(P, starts, lens)
        assert np.array_equal(fedavg.packed_to_param(cs, cl, np.arange(len(plain_idx))), plain_idx)
