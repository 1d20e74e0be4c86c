"""Sample-selection packers of the paper (Section 3.3, Table 1) as host-side integer code.

They decide which examples share a packed row; the attention path only sees the resulting
position ids.  Used by the benchmark to reproduce, at kernel level, the shape of the paper's
sampler comparisons (Tables 4-6): how full the rows get and how fast the resulting packs run.

Every packer takes example lengths and a row capacity (tokens per row) and returns rows as lists
of (example index, length) in stream order; an example longer than the capacity is truncated to
it (Section 3.3 keeps such examples out of a pack by truncation to the maximum length).  A row's
unused tail is padding: `position_ids` gives it to one pad pseudo-example.
"""
from __future__ import annotations

from typing import List, Sequence, Tuple

import numpy as np

Row = List[Tuple[int, int]]


def _clip(lengths: Sequence[int], capacity: int) -> List[int]:
    if capacity <= 0:
        raise ValueError("capacity must be positive")
    out = []
    for L in lengths:
        if L <= 0:
            raise ValueError("example lengths must be positive")
        out.append(min(int(L), capacity))
    return out


def first_fit_decreasing(lengths: Sequence[int], capacity: int) -> List[Row]:
    """Multipack (Table 1): examples in order of decreasing length (ties by index), each into the
    first row that still has room, a new row if none has."""
    ls = _clip(lengths, capacity)
    order = sorted(range(len(ls)), key=lambda i: (-ls[i], i))
    rows: List[Row] = []
    free: List[int] = []
    for i in order:
        for r in range(len(rows)):
            if free[r] >= ls[i]:
                rows[r].append((i, ls[i]))
                free[r] -= ls[i]
                break
        else:
            rows.append([(i, ls[i])])
            free.append(capacity - ls[i])
    return rows


def _next_fit(order: Sequence[int], ls: Sequence[int], capacity: int) -> List[Row]:
    rows: List[Row] = []
    room = 0
    for i in order:
        if not rows or room < ls[i]:
            rows.append([])
            room = capacity
        rows[-1].append((i, ls[i]))
        room -= ls[i]
    return rows


def sorted_packing(lengths: Sequence[int], capacity: int) -> List[Row]:
    """SortedPacking (Table 1): examples sorted by decreasing length, rows filled in that order; a
    row is closed when the next example does not fit."""
    ls = _clip(lengths, capacity)
    return _next_fit(sorted(range(len(ls)), key=lambda i: (-ls[i], i)), ls, capacity)


def random_packing(lengths: Sequence[int], capacity: int, seed: int = 0) -> List[Row]:
    """RandomPacking (Table 1): examples in a seeded random order, rows filled in that order."""
    ls = _clip(lengths, capacity)
    order = np.random.default_rng(seed).permutation(len(ls)).tolist()
    return _next_fit(order, ls, capacity)


def stream_packing(lengths: Sequence[int], capacity: int) -> List[Row]:
    """FixedLengthPacking with position ids (Table 1): examples concatenated in the given order and
    chopped every `capacity` tokens; an example that crosses a row end is broken in two (both parts
    listed with the same index)."""
    rows: List[Row] = [[]]
    room = capacity
    for i, L in enumerate(lengths):
        if L <= 0:
            raise ValueError("example lengths must be positive")
        left = int(L)
        while left > 0:
            if room == 0:
                rows.append([])
                room = capacity
            take = min(left, room)
            rows[-1].append((i, take))
            room -= take
            left -= take
    return [r for r in rows if r]


def efficiency(rows: List[Row], capacity: int) -> float:
    """Real tokens / row slots."""
    return sum(L for r in rows for _, L in r) / float(len(rows) * capacity) if rows else 0.0


def row_lengths(rows: List[Row], capacity: int) -> List[List[int]]:
    """Example lengths per row with the unused tail appended as one pad pseudo-example, so that
    every row holds exactly `capacity` tokens."""
    out = []
    for r in rows:
        ls = [L for _, L in r]
        used = sum(ls)
        if used > capacity:
            raise ValueError("row over capacity")
        if used < capacity:
            ls.append(capacity - used)
        out.append(ls)
    return out


def position_ids(rows: List[Row], capacity: int) -> np.ndarray:
    """[R, capacity] int64 ids restarting at 0 in every example (and in the pad tail)."""
    return np.stack([np.concatenate([np.arange(L, dtype=np.int64) for L in ls])
                     for ls in row_lengths(rows, capacity)], axis=0)


PACKERS = {"ffd": first_fit_decreasing, "sorted": sorted_packing, "random": random_packing, "stream": stream_packing}
