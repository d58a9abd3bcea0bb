"""Pins for the mask selection (oracle side): the definition by counting, closed forms, ties."""
import numpy as np

from oracle import select


def _by_counting(s, k):
    """Element i is among the k most sensitive iff fewer than k elements precede it in the order
    (larger value first, lower index first among equals): O(P^2), no sort."""
    s = np.asarray(s, dtype=np.float64)
    P = len(s)
    out = np.zeros(P, dtype=bool)
    for i in range(P):
        ahead = int(np.sum(s > s[i])) + int(np.sum(s[:i] == s[i]))
        out[i] = ahead < k
    return out


def test_select_matches_the_counting_definition():
    rs = np.random.default_rng(0)
    for trial in range(30):
        P = int(rs.integers(1, 200))
        if trial % 3 == 0:
            s = rs.integers(0, 4, P).astype(np.float32)            # many ties
        elif trial % 3 == 1:
            s = np.abs(rs.normal(0, 1, P)).astype(np.float32)
            s[rs.integers(0, P, P // 3)] = 0.0                     # exact zeros, some negative zeros
            s[rs.integers(0, P, 3)] = -0.0
        else:
            s = rs.normal(0, 1, P).astype(np.float32)              # negative values too
        for ratio in (0.0, 0.1, 0.3, 0.5, 0.9, 1.0, float(rs.random())):
            k = select.select_count(P, ratio)
            m = select.select_top(s, ratio)
            assert m.sum() == k
            assert np.array_equal(m, _by_counting(s, k))


def test_select_closed_forms_and_rounding():
    P = 1000
    dec = np.arange(P, 0, -1).astype(np.float32)                   # strictly decreasing: the first k
    assert select.runs_of(select.select_top(dec, 0.25)) == [(0, 250)]
    inc = np.arange(P).astype(np.float32)                          # strictly increasing: the last k
    assert select.runs_of(select.select_top(inc, 0.25)) == [(750, 250)]
    const = np.full(P, 3.0, dtype=np.float32)                      # all equal: lowest indices
    assert select.runs_of(select.select_top(const, 0.1)) == [(0, 100)]
    assert select.runs_of(select.select_top(const, 0.0)) == [] and select.runs_of(select.select_top(const, 1.0)) == [(0, P)]
    # k = rint(p * P), ties to even
    assert select.select_count(10, 0.25) == 2 and select.select_count(10, 0.35) == 4 and select.select_count(10, 0.05) == 0
    # -0.0 equals +0.0: index decides
    z = np.array([-0.0, 0.0, -0.0, 0.0], dtype=np.float32)
    assert select.runs_of(select.select_top(z, 0.5)) == [(0, 2)]


def test_runs_of():
    assert select.runs_of([0, 1, 1, 0, 1, 0, 0, 1]) == [(1, 2), (4, 1), (7, 1)]
    assert select.runs_of([1, 1, 1]) == [(0, 3)] and select.runs_of([0, 0]) == [] and select.runs_of([]) == []
