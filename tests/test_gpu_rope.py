"""Rotary embedding on the GPU vs the oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2407_09105_amd import binding, workloads as wl
from tests.gpu_util import BF16_MAX_ABS, BF16_REL_L2, DEV, max_abs, rel_l2

pytestmark = pytest.mark.gpu


def _run(x_np, pos_np, dtype, base=10000.0, inverse=False, id_dtype=torch.int64, inplace=False):
    x = torch.from_numpy(x_np).to(DEV).to(dtype)
    pos = torch.from_numpy(pos_np).to(DEV).to(id_dtype)
    y = binding.rope_apply(x, pos, base, inverse, out=x if inplace else None)
    torch.cuda.synchronize()
    return y.float().cpu().numpy().astype(np.float64)


def _rel_l2(a, b):
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-30))


@pytest.mark.parametrize("shape", [(300, 4, 128), (77, 3, 64), (50, 2, 80), (33, 5, 6), (19, 1, 256), (1, 1, 2)])
@pytest.mark.parametrize("inverse", [False, True])
def test_fp32(shape, inverse):
    rng = np.random.default_rng(sum(shape))
    x = rng.standard_normal(shape).astype(np.float32)
    pos = rng.integers(0, 20000, size=shape[0])
    pos[0] = 0
    got = _run(x, pos, torch.float32, inverse=inverse)
    ref = oracle.rope(x, pos, inverse=inverse)
    assert _rel_l2(got, ref) <= 1e-6            # far inside the 1e-4 bar of the fp32 path
    assert np.max(np.abs(got - ref)) <= 2e-6 * max(1.0, np.max(np.abs(ref)))
    assert np.array_equal(got[0], x[0].astype(np.float64))   # position 0: identity, exactly


@pytest.mark.parametrize("shape", [(2049, 32, 128), (130, 8, 128), (64, 4, 80), (41, 2, 72), (9, 3, 10)])
def test_bf16(shape):
    rng = np.random.default_rng(sum(shape) + 1)
    x = wl.round_to_bf16(rng.standard_normal(shape).astype(np.float32))
    pos = rng.integers(0, 16384, size=shape[0])
    got = _run(x, pos, torch.bfloat16)
    ref = oracle.rope(x, pos)
    # the result is stored in bf16: half an ulp (2^-9 relative) of rounding on top of ~1e-7 arithmetic
    assert np.all(np.abs(got - ref) <= 2.0 ** -8 * np.abs(ref) + 1e-6)
    assert _rel_l2(got, ref) <= 3e-3


@pytest.mark.parametrize("shape", [(515, 8, 128), (64, 4, 80), (9, 3, 10)])
@pytest.mark.parametrize("inplace", [False, True])
def test_fp16(shape, inplace):
    rng = np.random.default_rng(sum(shape) + 2)
    x = wl.round_to_f16(rng.standard_normal(shape).astype(np.float32))
    pos = rng.integers(0, 16384, size=shape[0])
    got = _run(x, pos, torch.float16, inplace=inplace)
    ref = oracle.rope(x, pos)
    # stored in fp16: half an ulp (2^-11 relative; 2^-25 absolute below the normal range)
    assert np.all(np.abs(got - ref) <= 2.0 ** -10 * np.abs(ref) + 1e-6)
    assert _rel_l2(got, ref) <= 5e-4


def test_large_positions_int32_inplace_and_base():
    rng = np.random.default_rng(4)
    x = rng.standard_normal((64, 2, 32)).astype(np.float32)
    pos = np.concatenate([np.array([0, 1, 16383, 65535, 1_000_000, 2**31 - 1]), rng.integers(0, 2**31 - 1, size=58)])
    for base in (10000.0, 500000.0):
        got = _run(x, pos, torch.float32, base=base, id_dtype=torch.int32, inplace=True)
        ref = oracle.rope(x, pos, base=base)
        assert np.max(np.abs(got - ref)) <= 5e-6, base   # fp64 angle reduction keeps 2^31-size angles exact


def test_inverse_undoes_and_empty():
    rng = np.random.default_rng(6)
    x = torch.from_numpy(rng.standard_normal((100, 2, 64)).astype(np.float32)).to(DEV)
    pos = torch.from_numpy(rng.integers(0, 9000, size=100)).to(DEV)
    y = binding.rope_apply(x, pos)
    back = binding.rope_apply(y, pos, inverse=True)
    assert torch.allclose(back, x, atol=2e-6)
    e = binding.rope_apply(torch.empty((0, 2, 64), device=DEV), torch.empty(0, dtype=torch.int64, device=DEV))
    assert e.shape == (0, 2, 64)


def test_rope_then_attention_matches_oracle():
    # the same position ids drive the rotary phase and the mask: rope(Q), rope(K) -> packed attention
    w = wl.make_custom([[200, 57, 300, 83]], hq=4, hkv=2, d=128, dtype="bf16", seed=12)
    t = lambda a: torch.from_numpy(a).to(DEV).to(torch.bfloat16)
    pos = torch.from_numpy(w.position_ids).to(DEV)
    q, k, v = t(w.q), t(w.k), t(w.v)
    qr, kr = binding.rope_apply(q, pos.reshape(-1)), binding.rope_apply(k, pos.reshape(-1))
    seg = binding.pack_to_cu_seqlens(pos)
    o, _ = binding.varlen_attn_fwd(qr, kr, v, seg)
    torch.cuda.synchronize()
    ref_seg = oracle.pack(w.position_ids)
    rq = wl.round_to_bf16(oracle.rope(w.q, w.position_ids).astype(np.float32))
    rk = wl.round_to_bf16(oracle.rope(w.k, w.position_ids).astype(np.float32))
    O_ref, _ = oracle.fwd(rq, rk, w.v, ref_seg["cu_seqlens"])
    got = o.float().cpu().numpy().astype(np.float64)
    # bf16 bar of the attention path; a rotated element whose fp32 and fp64 values round to different
    # bf16 neighbours moves one input by one ulp, far below it
    assert max_abs(got, O_ref) <= BF16_MAX_ABS and rel_l2(got, O_ref) <= BF16_REL_L2
