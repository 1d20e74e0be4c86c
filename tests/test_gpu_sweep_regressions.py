"""Regression cases from a wide seeded sweep of random shapes (rows up to 3000 tokens, 1-3 KV heads,
1-5 query heads per KV head, nine head dims, bf16 / fp16).

The fifteen seeds below are the ones that missed the stated bar (max-abs 2e-2, relative L2 5e-3 on
fp32-emitted gradients) before the backward carried its large probabilities and score gradients in
two bf16 parts and took D from the row sums of dS: fourteen with a dK (one also a dQ) entry of
2.0e-2 .. 2.6e-2 - all bf16 with 4 or 5 query heads per KV head - and one two-token input whose
only non-trivial row has a nearly one-hot softmax, where D = dO . O from the rounded O was off by
5 % of the tiny dQ and dK.  A few neighbours of the sweep run beside them.
"""
import numpy as np
import pytest
import torch

from paper_2407_09105_amd import workloads as wl
from tests.gpu_util import assert_close, assert_seg_equal, run_gpu, run_oracle

pytestmark = pytest.mark.gpu

MISSED = [5, 32, 33, 59, 91, 116, 118, 120, 143, 148, 170, 176, 191, 237, 247]
NEIGHBOURS = [0, 1, 58, 117, 142, 144, 236, 248]


def sweep_case(seed: int):
    rng = np.random.default_rng(5000 + seed)
    R = int(rng.integers(1, 4))
    T = int(rng.integers(1, int(rng.choice([300, 700, 1500, 3000]))))
    rows = []
    for _ in range(R):
        row, left = [], T
        while left > 0:
            L = int(min(left, rng.integers(1, max(2, int(rng.choice([8, 70, 300, 700, 3000]))))))
            row.append(L)
            left -= L
        rows.append(row)
    hkv = int(rng.choice([1, 2, 3]))
    hq = hkv * int(rng.choice([1, 2, 4, 5]))
    d = int(rng.choice([64, 96, 128, 40, 256, 160, 72, 112, 8]))
    dtype = str(rng.choice(["bf16", "f16"]))
    return wl.make_custom(rows, hq, hkv, d, dtype, seed=7000 + seed)


@pytest.mark.parametrize("seed", MISSED + NEIGHBOURS)
def test_sweep_seed_meets_the_stated_bar(seed):
    w = sweep_case(seed)
    print(f"case: sweep seed {seed} R={w.cfg.rows} T={w.cfg.tokens_per_row} hq={w.cfg.hq} hkv={w.cfg.hkv} "
          f"d={w.cfg.d} {w.cfg.dtype}", flush=True)
    got = run_gpu(w, grad_dtype=torch.float32, nan_fill=True)
    ref = run_oracle(w)
    assert_seg_equal(got["seg"], ref["seg"])
    assert_close(got, ref, w.cfg.dtype)


# Short-context queries (the first few tokens of an example) are where the rounding of the stored O
# shows most in dQ: D = dO . O is off by 2^-9 |dO . O| and the few probabilities are large.  The dQ kernel
# corrects them after its loop from key blocks that are still in LDS; two layouts had escaped it and sat
# at 0.9e-2 .. 1.6e-2 (inside the stated 2e-2, far above everything else in the tensor):
#   - packed rows that do not start on a multiple of 64 tokens (T % 64 != 0): key blocks were counted
#     from token 0, so a tile's own rows straddled three blocks and the first was gone by then;
#   - a tile whose first row belongs to an example that began a few tokens before the tile.
# The bound below is what the corrected rows reach.
SHORT_CONTEXT = [3119, 3093, 3055, 3128, 3142]
# head_dim 8 (softmax scale 0.35: the same error in D weighs four times what it does at head_dim 128) with a
# probability peak dozens of keys back: 1.0e-2 .. 1.4e-2 before head dims up to 32 kept the whole correction
SMALL_HEAD_DIM = [3356, 3043, 3395]


@pytest.mark.parametrize("seed", SHORT_CONTEXT + SMALL_HEAD_DIM)
def test_short_context_rows_are_corrected(seed):
    w = sweep_case(seed)
    print(f"case: sweep seed {seed} R={w.cfg.rows} T={w.cfg.tokens_per_row} hq={w.cfg.hq} hkv={w.cfg.hkv} "
          f"d={w.cfg.d} {w.cfg.dtype}", flush=True)
    got = run_gpu(w, grad_dtype=torch.float32, nan_fill=True)
    ref = run_oracle(w)
    assert_close(got, ref, w.cfg.dtype)
    err = float(np.abs(got["dQ"] - ref["dQ"]).max())
    print(f"   dQ max-abs {err:.2e}", flush=True)
    assert err <= 6e-3


@pytest.mark.parametrize("rows", [[[120, 48]], [[60, 70, 38]], [[125, 3, 40]], [[100, 100], [7, 193]], [[190, 66]]])
def test_short_context_rows_at_ragged_tiles(rows):
    # the same correction where a packed row ends with a tile of at most 64 rows (the keys before the tile
    # are then still in their stage) and where rows start off a multiple of 64
    w = wl.make_custom(rows, 4, 2, 128, "bf16", seed=77)
    got = run_gpu(w, grad_dtype=torch.float32, nan_fill=True)
    ref = run_oracle(w)
    assert_close(got, ref, "bf16")
    err = float(np.abs(got["dQ"] - ref["dQ"]).max())
    print(f"   dQ max-abs {err:.2e}", flush=True)
    assert err <= 6e-3
