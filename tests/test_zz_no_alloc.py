"""The backward entry point that allocates nothing (its D workspace is a device array inside the
library) against the ordinary backward, through the C ABI: two calls in a row, the second on a
smaller input, so that what the first call left in the shared array is still there."""
import pytest
import torch

from paper_2407_09105_amd import binding, workloads as wl
from tests.gpu_util import DEV, to_dev

pytestmark = pytest.mark.gpu


def _inputs(lengths, hq, hkv, d, dtype, seed):
    w = wl.make_custom(lengths, hq, hkv, d, dtype, seed=seed)
    q, k, v, do = (to_dev(a, dtype) for a in (w.q, w.k, w.v, w.do))
    seg = binding.pack_to_cu_seqlens(torch.from_numpy(w.position_ids).to(DEV))
    o, lse = binding.varlen_attn_fwd(q, k, v, seg)
    return q, k, v, do, o, lse, seg


def _both(lengths, hq, hkv, d, dtype, seed, grad_dtype):
    q, k, v, do, o, lse, seg = _inputs(lengths, hq, hkv, d, dtype, seed)
    ref = binding.varlen_attn_bwd(do, q, k, v, o, lse, seg, grad_dtype=grad_dtype)
    outs = [torch.full_like(r, float("nan")) for r in ref]
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    binding.varlen_attn_bwd_noalloc(do, q, k, v, o, lse, seg, *outs)
    assert torch.cuda.memory_allocated() == before       # no tensor was created on the way
    torch.cuda.synchronize()
    for name, a, b in zip(("dQ", "dK", "dV"), outs, ref):
        assert bool(torch.isfinite(a).all()), name
        assert torch.equal(a, b), name                   # same kernels, same order: bit for bit


def test_noalloc_backward_matches_backward_twice_in_a_row():
    # MFMA path (D formed by the dQ kernel), 3 rows of 1900 tokens, grouped heads
    _both([[700, 1200], [1900], [5] * 380], 8, 2, 128, "bf16", 61, torch.float32)
    # smaller input right after: fewer tokens and heads, 16-bit gradients; the array still holds the first call's D
    _both([[100, 219]], 2, 2, 64, "bf16", 62, torch.bfloat16)
    # plain kernels (fp32 inputs): D comes from the stand-alone D kernel
    _both([[40, 7, 81]], 4, 2, 40, "f32", 63, torch.float32)


def test_noalloc_backward_rejects_sizes_beyond_its_array():
    # N * Hq * 4 bytes of D must fit the library's array; validation happens before any launch
    rows, T, hq = 1, 70000, 128                        # 35.8 MB of D > 32 MiB
    assert rows * T * hq * 4 > binding.NOALLOC_SCRATCH_BYTES
    seg = binding.Segments(rows, T, DEV)
    binding.pack_to_cu_seqlens(torch.zeros((rows, T), dtype=torch.int32, device=DEV), seg)
    tiny = torch.zeros(8, device=DEV, dtype=torch.bfloat16)   # never dereferenced: the call is refused
    import ctypes as C
    st = binding.lib().va_varlen_attn_bwd_noalloc(
        *([tiny.data_ptr()] * 9), binding.VA_BF16, C.byref(seg.c), rows, T, hq, hq, 8, binding.VA_BF16, 0.0, None)
    assert st == 4                                      # VA_ERR_WORKSPACE
    torch.cuda.synchronize()
