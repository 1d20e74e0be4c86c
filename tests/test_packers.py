"""Host-side packers (Section 3.3, Table 1): invariants, hand-worked cases, and first-fit-decreasing
against the optimal number of rows found by brute force on small instances."""
import itertools

import numpy as np
import pytest

from oracle import oracle
from paper_2407_09105_amd import packers as pk


def _placed(rows):
    return sorted(i for r in rows for i, _ in r)


def test_ffd_hand_example():
    # capacity 10, lengths 7 5 4 3 2 2 1: decreasing order 7,5,4,3,2,2,1
    # 7 -> row0; 5 -> row1; 4 -> row1 (9); 3 -> row0 (10); 2 -> row2; 2 -> row2; 1 -> row1 (10)
    rows = pk.first_fit_decreasing([7, 5, 4, 3, 2, 2, 1], 10)
    assert rows == [[(0, 7), (3, 3)], [(1, 5), (2, 4), (6, 1)], [(4, 2), (5, 2)]]
    assert pk.efficiency(rows, 10) == 24 / 30


def test_sorted_and_stream_hand_examples():
    rows = pk.sorted_packing([3, 9, 4, 6, 2], 10)          # order 9,6,4,3,2 -> [9] [6,4] [3,2]
    assert rows == [[(1, 9)], [(3, 6), (2, 4)], [(0, 3), (4, 2)]]
    rows = pk.stream_packing([4, 8, 5, 11], 10)             # the worked example's lengths, rows of 10
    assert rows == [[(0, 4), (1, 6)], [(1, 2), (2, 5), (3, 3)], [(3, 8)]]
    assert pk.position_ids(rows, 10)[1].tolist() == [0, 1, 0, 1, 2, 3, 4, 0, 1, 2]
    assert pk.row_lengths(rows, 10)[2] == [8, 2]            # 2 pad tokens at the end of the last row


@pytest.mark.parametrize("name", ["ffd", "sorted", "random"])
@pytest.mark.parametrize("seed", range(5))
def test_invariants(name, seed):
    rng = np.random.default_rng(seed)
    cap = int(rng.integers(20, 400))
    lengths = rng.integers(1, int(cap * 1.3), size=int(rng.integers(1, 200))).tolist()
    rows = pk.PACKERS[name](lengths, cap)
    assert _placed(rows) == list(range(len(lengths)))                       # every example exactly once
    for r in rows:
        assert 0 < sum(L for _, L in r) <= cap
        assert all(L == min(lengths[i], cap) for i, L in r)                  # whole (or truncated) examples
    pos = pk.position_ids(rows, cap)
    assert pos.shape == (len(rows), cap)
    seg = oracle.pack(pos)                                                   # the ids give the rows' examples back
    assert np.diff(seg["cu_seqlens"]).tolist() == [L for ls in pk.row_lengths(rows, cap) for L in ls]
    if name == "sorted":
        flat = [L for r in rows for _, L in r]
        assert flat == sorted(flat, reverse=True)
    if name == "random":
        assert rows == pk.random_packing(lengths, cap, seed=0) and rows != pk.random_packing(lengths, cap, seed=1) or len(lengths) < 3


def _optimal_rows(ls, cap):
    # brute force: smallest k such that some assignment of examples to k rows fits
    n = len(ls)
    for k in range(1, n + 1):
        for assign in itertools.product(range(k), repeat=n):
            load = [0] * k
            for i, a in enumerate(assign):
                load[a] += ls[i]
            if max(load) <= cap:
                return k
    return n


@pytest.mark.parametrize("seed", range(12))
def test_ffd_against_brute_force_optimum(seed):
    rng = np.random.default_rng(50 + seed)
    cap = 20
    ls = rng.integers(1, 15, size=int(rng.integers(2, 8))).tolist()
    opt = _optimal_rows(ls, cap)
    got = len(pk.first_fit_decreasing(ls, cap))
    assert opt <= got <= (11 * opt) // 9 + 1                                 # the classical FFD guarantee
    assert got >= -(-sum(ls) // cap)


def test_errors():
    with pytest.raises(ValueError):
        pk.first_fit_decreasing([3, 0], 10)
    with pytest.raises(ValueError):
        pk.sorted_packing([3], 0)
