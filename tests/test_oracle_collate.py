"""Pins for the oracle's padding-free collator (Section 3.4 of the paper)."""
import numpy as np
import pytest

from oracle import oracle
from paper_2407_09105_amd import workloads as wl


def _padded(examples, Lp=None, fill=-1):
    Lp = Lp or max(1, max((len(e) for e in examples), default=1))
    out = np.full((len(examples), Lp), fill, dtype=np.int64)
    for r, e in enumerate(examples):
        out[r, : len(e)] = e
    return out


def _examples_of_worked_example(we):
    ids, out, t = we["input_ids"], [], 0
    for L in we["lengths"]:
        out.append(ids[t : t + L])
        t += L
    return out


def test_paper_worked_example(worked_example):
    # Section 3.5: four sequences [10..13], [20..27], [30..34], [40..49, 410]; the paper prints
    # the collator's input_ids, labels and position_ids.
    ex = _examples_of_worked_example(worked_example)
    assert ex[0] == [10, 11, 12, 13] and ex[3][-1] == 410
    out = oracle.collate(_padded(ex), worked_example["lengths"], 28)
    assert out["input_ids"].tolist() == worked_example["input_ids"]
    assert out["labels"].tolist() == worked_example["labels"]
    assert out["position_ids"].tolist() == worked_example["position_ids"]
    assert out["offsets"].tolist() == worked_example["cu_seqlens"]


def test_three_rules_by_hand():
    # written out independently with numpy: concatenate, first label -> -100, arange per example
    rng = np.random.default_rng(5)
    lengths = [int(x) for x in rng.integers(1, 30, size=17)]
    ex = [rng.integers(0, 32000, size=L).tolist() for L in lengths]
    lab = [rng.integers(0, 32000, size=L).tolist() for L in lengths]
    N = sum(lengths)
    out = oracle.collate(_padded(ex), lengths, N, labels_padded=_padded(lab))
    assert out["input_ids"].tolist() == sum(ex, [])
    expect_lab = np.concatenate([np.array(l) for l in lab])
    starts = np.cumsum([0] + lengths[:-1])
    expect_lab[starts] = -100
    assert out["labels"].tolist() == expect_lab.tolist()
    assert out["position_ids"].tolist() == np.concatenate([np.arange(L) for L in lengths]).tolist()
    assert out["offsets"].tolist() == np.cumsum([0] + lengths).tolist()
    # labels default to the ids
    out2 = oracle.collate(_padded(ex), lengths, N)
    e2 = np.array(sum(ex, []))
    e2[starts] = -100
    assert out2["labels"].tolist() == e2.tolist()


@pytest.mark.parametrize("seed", range(6))
def test_ids_give_the_lengths_back(seed):
    # the collator's position ids, fed to the boundary scan, return the example lengths
    rng = np.random.default_rng(100 + seed)
    lengths = [int(x) for x in rng.integers(1, 50, size=int(rng.integers(1, 40)))]
    ex = [list(range(1000 * i, 1000 * i + L)) for i, L in enumerate(lengths)]
    N = sum(lengths)
    out = oracle.collate(_padded(ex), lengths, N)
    seg = oracle.pack(out["position_ids"][None, :])
    assert np.diff(seg["cu_seqlens"]).tolist() == lengths
    assert seg["cu_seqlens"].tolist() == out["offsets"].tolist()
    # and they are the ids of the shared workload generator
    assert out["position_ids"].tolist() == wl.position_ids_from_lengths([lengths])[0].tolist()
    # every token of example i sits where the offsets say
    for i, L in enumerate(lengths):
        assert out["input_ids"][out["offsets"][i] : out["offsets"][i + 1]].tolist() == ex[i]


def test_tail_and_cut_and_clamp():
    ex = [[1, 2, 3], [4, 5], [6, 7, 8, 9]]
    pad = _padded(ex, Lp=4, fill=-5)
    # short sum: pad pseudo-example at the tail
    out = oracle.collate(pad, [3, 2, 4], 12, pad_id=77)
    assert out["input_ids"].tolist() == [1, 2, 3, 4, 5, 6, 7, 8, 9, 77, 77, 77]
    assert out["labels"].tolist() == [-100, 2, 3, -100, 5, -100, 7, 8, 9, -100, -100, -100]
    assert out["position_ids"].tolist() == [0, 1, 2, 0, 1, 0, 1, 2, 3, 0, 1, 2]
    # long sum: cut at n_out, offsets still the full running sum
    out = oracle.collate(pad, [3, 2, 4], 7)
    assert out["input_ids"].tolist() == [1, 2, 3, 4, 5, 6, 7]
    assert out["position_ids"].tolist() == [0, 1, 2, 0, 1, 0, 1]
    assert out["offsets"].tolist() == [0, 3, 5, 9]
    # clamped lengths, empty examples
    out = oracle.collate(pad, [9, -3, 0], 5, pad_id=0)
    assert out["input_ids"].tolist() == [1, 2, 3, -5, 0]
    assert out["position_ids"].tolist() == [0, 1, 2, 3, 0]
    assert out["offsets"].tolist() == [0, 4, 4, 4]
    # no examples at all
    out = oracle.collate(np.zeros((0, 4), dtype=np.int64), np.zeros(0, dtype=np.int32), 3, pad_id=9)
    assert out["input_ids"].tolist() == [9, 9, 9] and out["position_ids"].tolist() == [0, 1, 2]
