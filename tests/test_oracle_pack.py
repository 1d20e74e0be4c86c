"""Pins for the oracle's boundary extraction (position_ids -> cu_seqlens)."""
import numpy as np
import pytest

from oracle import oracle
from paper_2407_09105_amd import workloads as wl


def test_paper_worked_example(worked_example):
    # Section 3.5 of the paper: lengths 4, 8, 5, 11; ids as printed there.
    pos = np.array([worked_example["position_ids"]], dtype=np.int64)
    out = oracle.pack(pos)
    assert out["cu_seqlens"].tolist() == worked_example["cu_seqlens"] == [0, 4, 12, 17, 28]
    assert out["n"] == 4
    assert out["max_seqlen"] == worked_example["max_seqlen"][0] == 11
    assert np.diff(out["cu_seqlens"]).tolist() == worked_example["lengths"]
    # segment ids: token t belongs to the example whose [cu[s], cu[s+1]) holds it
    expect = sum(([s] * L for s, L in enumerate(worked_example["lengths"])), [])
    assert out["seg_id"].tolist() == expect


def test_generator_reproduces_worked_example_ids(worked_example):
    # the generator's ids for lengths 4, 8, 5, 11 are the ones the paper prints
    pos = wl.position_ids_from_lengths([worked_example["lengths"]])
    assert pos[0].tolist() == worked_example["position_ids"]


def test_config1_ids_and_cu():
    w = wl.make_workload(1, tensors=False)
    assert w.position_ids[0].tolist() == [0, 1, 2, 0, 1, 2, 3, 4, 0, 0, 1, 2, 3, 4, 5, 6]
    out = oracle.pack(w.position_ids)
    assert out["cu_seqlens"].tolist() == [0, 3, 8, 9, 16]
    assert out["n"] == 4 and out["max_seqlen"] == 7
    assert out["seg_id"].tolist() == [0] * 3 + [1] * 5 + [2] + [3] * 7


@pytest.mark.parametrize("seed", range(8))
def test_roundtrip_lengths(seed):
    rng = np.random.default_rng(seed)
    R = int(rng.integers(1, 4))
    T = int(rng.integers(1, 200))
    rows = []
    for _ in range(R):
        row, left = [], T
        while left > 0:
            L = int(rng.integers(1, min(left, 40) + 1))
            row.append(L)
            left -= L
        rows.append(row)
    pos = wl.position_ids_from_lengths(rows)
    out = oracle.pack(pos)
    flat = [L for row in rows for L in row]
    assert np.diff(out["cu_seqlens"]).tolist() == flat
    assert out["n"] == len(flat) and out["max_seqlen"] == max(flat)
    assert out["cu_seqlens"][0] == 0 and out["cu_seqlens"][-1] == R * T
    # seg_start / seg_end bracket each token
    t = np.arange(R * T)
    assert np.all(out["seg_start"] <= t) and np.all(t < out["seg_end"])
    assert np.all(out["seg_end"] - out["seg_start"] == np.repeat(flat, flat))


def test_row_start_is_always_a_boundary():
    # second row starts with a non-zero id (an example continued from the row before):
    # rows are separate batch elements, so it still starts a segment
    pos = np.array([[0, 1, 2, 3, 0, 1], [5, 6, 7, 0, 1, 2]], dtype=np.int64)
    out = oracle.pack(pos)
    assert out["cu_seqlens"].tolist() == [0, 4, 6, 9, 12]
    assert out["seg_id"].tolist() == [0, 0, 0, 0, 1, 1, 2, 2, 2, 3, 3, 3]


def test_consecutive_zeros_are_length_one_examples():
    pos = np.array([[0, 1, 2, 0, 0, 0, 1]], dtype=np.int64)
    out = oracle.pack(pos)
    assert out["cu_seqlens"].tolist() == [0, 3, 4, 5, 7]
    assert out["max_seqlen"] == 3


def test_only_zero_marks_a_boundary():
    # a jump that is not a restart at 0 does not split; negative ids do not split
    pos = np.array([[0, 1, 7, 8, 3, -1, 0, 1]], dtype=np.int64)
    out = oracle.pack(pos)
    assert out["cu_seqlens"].tolist() == [0, 6, 8]


def test_single_token_and_single_segment():
    assert oracle.pack(np.array([[0]]))["cu_seqlens"].tolist() == [0, 1]
    out = oracle.pack(np.arange(37, dtype=np.int64)[None, :])
    assert out["cu_seqlens"].tolist() == [0, 37] and out["n"] == 1 and out["max_seqlen"] == 37
