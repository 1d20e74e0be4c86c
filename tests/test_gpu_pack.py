"""GPU boundary scan vs the oracle: bit-exact (integer work)."""
import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2407_09105_amd import binding, workloads as wl
from tests.gpu_util import DEV, assert_seg_equal

pytestmark = pytest.mark.gpu


def _gpu_pack(pos_np, dtype=torch.int64):
    pos = torch.from_numpy(pos_np).to(DEV).to(dtype)
    seg = binding.pack_to_cu_seqlens(pos)
    torch.cuda.synchronize()
    return seg.host()


def _check_orders(got, pos_np):
    R, T = pos_np.shape
    ref = oracle.pack(pos_np)
    TILE = binding.VA_TILE
    tpr = (T + TILE - 1) // TILE
    nt = R * tpr
    tiles = np.arange(nt)
    t0 = (tiles // tpr) * T + (tiles % tpr) * TILE
    t1 = np.minimum(t0 + TILE, (tiles // tpr + 1) * T) - 1
    ss, se = ref["seg_start"].astype(np.int64), ref["seg_end"].astype(np.int64)
    cost_q = (t1 >> 6) - (ss[t0] >> 6) + 1
    cost_kv = ((se[t1] - 1) >> 6) - (t0 >> 6) + 1

    def key(length, start, cost):
        # examples of at most one schedule tile all rank alike (they stay in stream order), longer ones by length
        rank = np.where(length <= TILE, 0, np.minimum(length, (1 << 20) - 1))
        return (rank << 43) | ((0x7FFFFFFF - start) << 12) | np.minimum(cost, 4095)

    key_q = key(se[t0] - ss[t0], ss[t0], cost_q)       # governed by the example of the tile's first token
    key_kv = key(se[t1] - ss[t1], ss[t1], cost_kv)     # ... of its last token
    for name, k, cost in (("q_tile_order", key_q, cost_q), ("kv_tile_order", key_kv, cost_kv)):
        order = got[name]
        assert sorted(order.tolist()) == list(range(nt)), name     # a permutation of the tiles
        assert np.all(cost >= 1)
        # largest key first, ties keep index order: the result is unique
        expect = np.lexsort((tiles, -k))
        assert np.array_equal(order, expect), name
    # Design properties of the schedule, stated without the sort key: tiles governed by examples longer
    # than a schedule tile come first, longest example first, the tiles of one example adjacent and
    # sharing one head rotation; tiles of shorter examples follow in stream order, rotation = rank / 8.
    for name, rot_name, gov in (("q_tile_order", "q_tile_rotation", t0), ("kv_tile_order", "kv_tile_rotation", t1)):
        order, rot = got[name], got[rot_name]
        glen = (se[gov] - ss[gov])[order]          # length of each tile's governing example, in launch order
        gstart = ss[gov][order]
        long_ = glen > TILE
        n_long = int(long_.sum())
        assert long_[:n_long].all() and not long_[n_long:].any()
        assert np.all(np.diff(glen[:n_long]) <= 0)                       # longest first
        runs = np.flatnonzero(np.diff(gstart[:n_long]) != 0) + 1         # where the governing example changes
        assert len(set(gstart[:n_long].tolist())) == len(runs) + (1 if n_long else 0)   # one run per example: adjacent
        for a, b in zip(np.r_[0, runs], np.r_[runs, n_long]) if n_long else ():
            assert len(set(rot[a:b].tolist())) == 1                      # one rotation per long example
        assert np.array_equal(order[n_long:], np.sort(order[n_long:]))   # short ones: stream order
        assert np.array_equal(rot[n_long:], (np.arange(n_long, nt) >> 3) & 127)


def test_worked_example(worked_example):
    pos = np.array([worked_example["position_ids"]], dtype=np.int64)
    got = _gpu_pack(pos)
    assert got["cu_seqlens"].tolist() == worked_example["cu_seqlens"]
    assert got["n"] == 4 and got["max_seqlen"] == 11
    assert_seg_equal(got, oracle.pack(pos))


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
@pytest.mark.parametrize("dtype", [torch.int64, torch.int32])
def test_configs(cfg, dtype):
    w = wl.make_workload(cfg, tensors=False)
    got = _gpu_pack(w.position_ids, dtype)
    assert_seg_equal(got, oracle.pack(w.position_ids))
    _check_orders(got, w.position_ids)


@pytest.mark.parametrize("R,T,maxlen,seed", [
    (1, 1, 1, 0), (1, 7, 3, 1), (3, 129, 40, 2), (2, 2048, 300, 3), (5, 2049, 17, 4),
    (1, 4097, 5000, 5), (7, 1000, 1, 6), (2, 70001, 900, 7), (1, 300000, 2500, 8),
    (1, 8192, 8192, 9), (2, 4096, 700, 10), (1, 8193, 600, 11),   # around the one-launch limit (8192 tokens)
    (300, 20, 20, 12), (2000, 4, 3, 13),                          # <= 8192 tokens but more than 256 tiles
    (3000, 5, 4, 14),                                             # more than 2048 tiles: separate key / rank kernels
])
def test_ragged_shapes(R, T, maxlen, seed):
    rng = np.random.default_rng(seed)
    rows = []
    for _ in range(R):
        row, left = [], T
        while left > 0:
            L = int(rng.integers(1, min(left, maxlen) + 1))
            row.append(L)
            left -= L
        rows.append(row)
    pos = wl.position_ids_from_lengths(rows)
    got = _gpu_pack(pos)
    assert_seg_equal(got, oracle.pack(pos))
    _check_orders(got, pos)


def test_rows_not_starting_at_zero_and_odd_ids():
    pos = np.array([[0, 1, 2, 3, 0, 1], [5, 6, 7, 0, 1, 2], [3, 3, 3, 3, -1, 9]], dtype=np.int64)
    got = _gpu_pack(pos)
    assert got["cu_seqlens"].tolist() == [0, 4, 6, 9, 12, 18]
    assert_seg_equal(got, oracle.pack(pos))


def test_pack_twice_into_same_plan():
    # the plan buffer is reusable: a second pack overwrites every field
    w4 = wl.make_workload(4, tensors=False)
    pos_a = torch.from_numpy(w4.position_ids).to(DEV)
    seg = binding.pack_to_cu_seqlens(pos_a)
    one = np.tile(np.arange(8192, dtype=np.int64), (8, 1))
    binding.pack_to_cu_seqlens(torch.from_numpy(one).to(DEV), seg)
    torch.cuda.synchronize()
    assert_seg_equal(seg.host(), oracle.pack(one))
