"""Device-side padding-free collator vs the oracle: bit-exact (integer work), through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2407_09105_amd import binding, workloads as wl
from tests.gpu_util import DEV

pytestmark = pytest.mark.gpu


def _padded(examples, Lp, fill=-1):
    out = np.full((len(examples), Lp), fill, dtype=np.int64)
    for r, e in enumerate(examples):
        out[r, : len(e)] = e
    return out


def _gpu(ids, lengths, n_out, labels=None, pad_id=0, dtype=torch.int64):
    t = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(DEV).to(dtype)
    out = binding.collate_padding_free(t(ids), torch.tensor(lengths, dtype=torch.int32, device=DEV).reshape(-1),
                                       n_out, labels_padded=t(labels), pad_id=pad_id)
    torch.cuda.synchronize()
    return {k: v.cpu().numpy() for k, v in out.items()}


def _compare(ids, lengths, n_out, labels=None, pad_id=0, dtype=torch.int64):
    got = _gpu(ids, lengths, n_out, labels, pad_id, dtype)
    ref = oracle.collate(ids, lengths, n_out, labels_padded=labels, pad_id=pad_id)
    for k in ("input_ids", "labels", "position_ids"):
        assert got[k].shape == (1, n_out)
        assert np.array_equal(got[k][0].astype(np.int64), ref[k]), k
    assert np.array_equal(got["example_offsets"], ref["offsets"])
    return got


def test_paper_worked_example(worked_example):
    # Section 3.5: the three tensors the paper prints, from the device collator
    ex, t = [], 0
    for L in worked_example["lengths"]:
        ex.append(worked_example["input_ids"][t : t + L])
        t += L
    got = _gpu(_padded(ex, 11), worked_example["lengths"], 28)
    assert got["input_ids"][0].tolist() == worked_example["input_ids"]
    assert got["labels"][0].tolist() == worked_example["labels"]
    assert got["position_ids"][0].tolist() == worked_example["position_ids"]
    assert got["example_offsets"].tolist() == worked_example["cu_seqlens"]


@pytest.mark.parametrize("dtype", [torch.int64, torch.int32])
@pytest.mark.parametrize("seed", range(4))
def test_random_batches(seed, dtype):
    rng = np.random.default_rng(300 + seed)
    n = int(rng.integers(1, 3000))
    Lp = int(rng.integers(1, 300))
    lengths = rng.integers(0 if seed % 2 else 1, Lp + 1, size=n).astype(np.int32)
    ids = rng.integers(0, 2**31 - 1, size=(n, Lp))
    labels = rng.integers(-100, 2**31 - 1, size=(n, Lp)) if seed >= 2 else None
    total = int(lengths.sum())
    _compare(ids, lengths, total, labels, dtype=dtype)


def test_tail_cut_clamp_and_empty():
    rng = np.random.default_rng(9)
    n, Lp = 700, 37
    lengths = rng.integers(-5, Lp + 9, size=n).astype(np.int32)       # some outside [0, Lp]
    ids = rng.integers(0, 50000, size=(n, Lp))
    total = int(np.clip(lengths, 0, Lp).sum())
    _compare(ids, lengths, total + 1000, pad_id=11)                    # pad pseudo-example at the tail
    _compare(ids, lengths, total - 999)                                # cut inside an example
    _compare(ids, lengths, 1)
    _compare(ids, np.zeros(n, dtype=np.int32), 50, pad_id=3)           # only empty examples
    _compare(np.zeros((0, 4), dtype=np.int64), np.zeros(0, dtype=np.int32), 19, pad_id=5)  # no examples
    got = _gpu(ids, lengths, 0)
    assert got["example_offsets"][-1] == total


def test_feeds_the_boundary_scan():
    # collator -> position ids -> va_pack_to_cu_seqlens gives the example offsets back
    # (no empty examples: an empty example has no token to carry a 0)
    w = wl.make_workload(3, tensors=False)
    lengths = np.array(w.lengths[0], dtype=np.int32)
    n, Lp = len(lengths), int(lengths.max())
    rng = np.random.default_rng(1)
    ids = rng.integers(0, 32000, size=(n, Lp))
    t = lambda a: torch.from_numpy(a).to(DEV)
    out = binding.collate_padding_free(t(ids), t(lengths), w.cfg.tokens_per_row)
    seg = binding.pack_to_cu_seqlens(out["position_ids"])
    torch.cuda.synchronize()
    h = seg.host()
    assert np.array_equal(h["cu_seqlens"], out["example_offsets"].cpu().numpy())
    assert np.array_equal(out["position_ids"].cpu().numpy(), w.position_ids[:1])
