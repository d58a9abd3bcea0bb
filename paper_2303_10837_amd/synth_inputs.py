"""Seeded synthetic workloads shared by the GPU tests, the benchmark and the CPU reference checks.

Holds no arithmetic of the method: only the shapes, value distributions and
mask structure of the five workloads (model-sized Gaussian parameter vectors,
client sample counts, block-structured selective-encryption masks).  The
paper evaluates on trained checkpoints (ResNet, BERT, ... ; Section "Results
on Different Scales of Models"); HE cost depends only on sizes (it is linear
in the number of encrypted parameters), so size-matched Gaussian vectors
stand in for them.

Importing this module never loads the HIP library.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

MASTER_SEED = 20230310


@dataclass(frozen=True)
class Workload:
    name: str
    index: int            # seed offset
    n_clients: int
    n_params: int
    log2_n: int
    n_limbs: int
    std: float            # parameter std (ignored when seg_std is set)
    enc_ratio: float      # 1.0 = fully encrypted
    block_lo: int = 0
    block_hi: int = 0
    seg_std: bool = False  # per-segment std drawn in [0.01, 0.05], whole segments masked
    scale_bits: int = 30
    cbd_eta: int = 21

    @property
    def seed(self) -> int:
        return MASTER_SEED + self.index


WORKLOADS = {
    "tiny_full": Workload("tiny_full", 1, 3, 100_000, 13, 3, 0.05, 1.0),
    "resnet18_full": Workload("resnet18_full", 2, 8, 11_700_000, 14, 4, 0.02, 1.0),
    "resnet50_sel10": Workload("resnet50_sel10", 3, 16, 25_600_000, 14, 4, 0.02, 0.10, 4096, 65536),
    "bert_sel10": Workload("bert_sel10", 4, 8, 110_000_000, 14, 4, 0.0, 0.10, 768, 589_824, True),
    "bert_full": Workload("bert_full", 4, 8, 110_000_000, 14, 4, 0.0, 1.0, 768, 589_824, True),
    "fm1p3b_sel5": Workload("fm1p3b_sel5", 5, 32, 1_300_000_000, 14, 4, 0.02, 0.05, 2048, 4_194_304),
}


def scaled(w: Workload, n_params: int, n_clients: int | None = None) -> Workload:
    """Same recipe at a smaller size (for quick tests); block sizes are kept."""
    from dataclasses import replace
    return replace(w, n_params=n_params, n_clients=n_clients or w.n_clients)


def client_alphas(w: Workload):
    """FedAvg weights: sample counts uniform in [100, 1000], normalised (float64)."""
    counts = np.random.default_rng([w.seed, 0xA1FA]).integers(100, 1001, size=w.n_clients)
    return counts.astype(np.float64) / np.float64(counts.sum())


def _segments(w: Workload):
    """Consecutive segments of length U{block_lo..block_hi} covering [0, P)."""
    rs = np.random.default_rng([w.seed, 0x5E65])
    bounds = [0]
    while bounds[-1] < w.n_params:
        bounds.append(min(w.n_params, bounds[-1] + int(rs.integers(w.block_lo, w.block_hi + 1))))
    return np.asarray(bounds, dtype=np.int64)


def mask_runs(w: Workload):
    """Sorted disjoint runs (starts, lens) as uint64 arrays; touching runs are merged."""
    P = w.n_params
    if w.enc_ratio >= 1.0:
        return np.array([0], dtype=np.uint64), np.array([P], dtype=np.uint64)
    target = int(round(w.enc_ratio * P))
    rs = np.random.default_rng([w.seed, 0x3A5C])
    runs = []
    if w.seg_std:
        b = _segments(w)
        order = rs.permutation(len(b) - 1)
        got = 0
        for s in order:
            if got >= target:
                break
            length = int(min(b[s + 1] - b[s], target - got))
            runs.append((int(b[s]), length))
            got += length
        runs.sort()
    else:
        lens = []
        while sum(lens) < target:
            lens.append(int(rs.integers(w.block_lo, w.block_hi + 1)))
        lens[-1] -= sum(lens) - target
        gap_total = P - target
        cuts = np.sort(rs.integers(0, gap_total + 1, size=len(lens)))
        pos = 0
        prev_cut = 0
        for ln, cut in zip(lens, cuts):
            pos += int(cut - prev_cut)
            prev_cut = int(cut)
            runs.append((pos, ln))
            pos += ln
    merged = []
    for s, ln in runs:
        if ln <= 0:
            continue
        if merged and merged[-1][0] + merged[-1][1] == s:
            merged[-1] = (merged[-1][0], merged[-1][1] + ln)
        else:
            merged.append((s, ln))
    starts = np.array([r[0] for r in merged], dtype=np.uint64)
    lens_a = np.array([r[1] for r in merged], dtype=np.uint64)
    return starts, lens_a


def _std_vector_segments(w: Workload):
    b = _segments(w)
    rs = np.random.default_rng([w.seed, 0x57D0])
    return b, rs.uniform(0.01, 0.05, size=len(b) - 1)


def client_params_numpy(w: Workload, client: int):
    """float32[P] on the host."""
    rs = np.random.default_rng([w.seed, 0xC11E, client])
    x = rs.standard_normal(w.n_params, dtype=np.float32)
    if w.seg_std:
        b, sd = _std_vector_segments(w)
        x *= np.repeat(sd.astype(np.float32), np.diff(b))
    else:
        x *= np.float32(w.std)
    return x


def client_params_torch(w: Workload, client: int, device):
    """float32[P] generated on `device` by torch's own seeded generator (for the
    sizes that are too slow to draw on the host).  Not bit-identical to the numpy
    variant; whoever needs the values on the host copies them back."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(w.seed * 1000 + client)
    x = torch.randn(w.n_params, generator=g, device=device, dtype=torch.float32)
    if w.seg_std:
        b, sd = _std_vector_segments(w)
        sdv = torch.repeat_interleave(torch.tensor(sd, dtype=torch.float32, device=device),
                                      torch.tensor(np.diff(b), device=device))
        x *= sdv
    else:
        x *= w.std
    return x
