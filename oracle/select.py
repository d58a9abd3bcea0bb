"""Encryption-mask agreement (oracle side): Select(global privacy map, p).

Algorithm 1 ("Server Encryption Mask Aggregation") forms the global privacy map
sum_i alpha_i [[S_i]] from the clients' encrypted sensitivity maps and configures
the mask M from it: a ratio p in [0, 1] says which share of the parameters, the
most sensitive ones, gets encrypted (Section "Selective Parameter Encryption",
Step 2).  The aggregation is the ordinary secure round with
everything encrypted; the selection works on the decrypted map (a comparison is
not a depth-1 homomorphic operation; the paper leaves open who decrypts).

Readings where the paper is silent: k = rint(p * P) parameters are selected
(ties to even, as for the aggregation weights); among equal sensitivities the
lower parameter index wins; -0.0 and +0.0 are equal; the map holds no NaN.
"""
from __future__ import annotations

import numpy as np


def select_count(P: int, ratio: float) -> int:
    return int(np.rint(np.float64(ratio) * np.float64(P)))


def select_top(sens, ratio: float):
    """Boolean mask (length P) of the k most sensitive parameters."""
    s = np.asarray(sens, dtype=np.float32).astype(np.float64)
    P = s.shape[0]
    k = select_count(P, ratio)
    mask = np.zeros(P, dtype=bool)
    if k > 0:
        order = np.lexsort((np.arange(P), -s))     # by sensitivity descending, then index ascending
        mask[order[:k]] = True
    return mask


def runs_of(mask):
    """Maximal runs (start, length) of a boolean mask, in order."""
    m = np.asarray(mask, dtype=bool)
    d = np.diff(np.concatenate([[0], m.astype(np.int8), [0]]))
    starts = np.flatnonzero(d == 1)
    ends = np.flatnonzero(d == -1)
    return [(int(a), int(b - a)) for a, b in zip(starts, ends)]
