"""What the parity suite would otherwise not look at: writes outside the output tensors, the
stand-alone D kernel, the plain kernels forced onto a shape the MFMA kernels normally take, and
packs made by the paper's samplers (pad tails, broken examples) through the whole path."""
import os
import subprocess
import sys

import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2407_09105_amd import binding, packers as pk, workloads as wl
from tests.gpu_util import DEV, assert_close, assert_seg_equal, rel_l2, run_gpu, run_oracle, to_dev

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _guarded(shapes_dtypes, guard_bytes=4096, pattern=0x5A):
    """One byte buffer holding the given tensors, each preceded and followed by `guard_bytes` of
    `pattern`; returns (views, check) where check() asserts every guard byte is untouched."""
    offs, off = [], guard_bytes
    for shape, dtype in shapes_dtypes:
        nbytes = int(np.prod(shape)) * torch.empty((), dtype=dtype).element_size()
        offs.append((off, nbytes))
        off += (nbytes + guard_bytes + 255) // 256 * 256
    buf = torch.full((off + guard_bytes,), pattern, dtype=torch.uint8, device=DEV)
    views, covered = [], torch.zeros_like(buf, dtype=torch.bool)
    for (o, nbytes), (shape, dtype) in zip(offs, shapes_dtypes):
        assert o % 16 == 0
        views.append(buf[o:o + nbytes].view(dtype).view(shape))
        covered[o:o + nbytes] = True

    def check():
        torch.cuda.synchronize()
        bad = (buf != pattern) & ~covered
        assert not bool(bad.any()), f"{int(bad.sum())} guard bytes overwritten, first at {int(bad.nonzero()[0])}"

    return views, check


@pytest.mark.parametrize("lengths,hq,hkv,d,dtype,gdt", [
    ([[100, 219], [319], [1] * 319], 2, 2, 128, "bf16", torch.float32),      # ragged T = 319
    ([[100, 219], [319], [1] * 319], 4, 2, 72, "bf16", torch.bfloat16),      # d = 72 < the 96 it is unrolled for
    ([[513, 31, 480, 7]], 5, 1, 8, "f16", torch.float16),                    # d = 8, G = 5, T = 1031
    ([[70, 1, 129, 1000, 33]], 2, 1, 200, "bf16", torch.float32),            # d = 200 in the 256 instantiation, T = 1233
    ([[1100, 1030, 1]], 2, 1, 128, "bf16", torch.bfloat16),                  # the dK/dV kernel's large shape, ragged last tile
    ([[9, 3, 20]], 2, 2, 20, "f32", torch.float32),                          # plain kernels
])
def test_nothing_is_written_outside_the_outputs(lengths, hq, hkv, d, dtype, gdt):
    w = wl.make_custom(lengths, hq, hkv, d, dtype, seed=77)
    N = w.cfg.n_tokens
    q, k, v, do = (to_dev(a, dtype) for a in (w.q, w.k, w.v, w.do))
    (o, lse, dq, dk, dv, ws), check = _guarded([
        ((N, hq, d), q.dtype), ((hq, N), torch.float32), ((N, hq, d), gdt), ((N, hkv, d), gdt), ((N, hkv, d), gdt),
        ((binding.lib().va_attn_workspace_bytes(N, hq, hkv, d, 1) // 4,), torch.float32)])
    seg = binding.pack_to_cu_seqlens(torch.from_numpy(w.position_ids).to(DEV))
    binding.varlen_attn_fwd(q, k, v, seg, out=o, lse=lse)
    binding.varlen_attn_bwd(do, q, k, v, o, lse, seg, dq=dq, dk=dk, dv=dv, workspace=ws)
    check()
    # and what was written inside is right
    ref = run_oracle(w)
    f = lambda t: t.float().cpu().numpy().astype(np.float64)
    got = {"O": f(o), "LSE": f(lse), "dQ": f(dq), "dK": f(dk), "dV": f(dv)}
    assert_close(got, ref, dtype, bf16_stored=("dQ", "dK", "dV") if gdt != torch.float32 else ())


def test_binding_refuses_output_buffers_the_library_would_overrun():
    # the library only gets pointers: a caller-supplied output of the wrong type, shape or layout must not reach it
    w = wl.make_custom([[40, 24]], 4, 2, 64, "bf16", seed=3)
    q, k, v, do = (to_dev(a, "bf16") for a in (w.q, w.k, w.v, w.do))
    seg = binding.pack_to_cu_seqlens(torch.from_numpy(w.position_ids).to(DEV))
    o, lse = binding.varlen_attn_fwd(q, k, v, seg)
    f32 = lambda t: torch.empty(t.shape, dtype=torch.float32, device=DEV)
    with pytest.raises(ValueError):
        binding.varlen_attn_fwd(q, k, v, seg, out=f32(q))                          # fp32 out for bf16 inputs
    with pytest.raises(ValueError):
        binding.varlen_attn_fwd(q, k, v, seg, lse=torch.empty((64, 4), dtype=torch.float32, device=DEV))   # transposed LSE
    with pytest.raises(ValueError):
        binding.varlen_attn_fwd(q, k, v, seg, out=torch.empty((64, 8, 64), dtype=q.dtype, device=DEV)[:, ::2])  # not contiguous
    with pytest.raises(ValueError):
        binding.varlen_attn_bwd(do, q, k, v, o, lse, seg, dq=f32(q), dk=f32(q), dv=f32(v))   # dK of dQ's shape under GQA
    with pytest.raises(ValueError):
        binding.varlen_attn_bwd(do, q, k, v, o, lse, seg, dq=f32(q), dk=torch.empty_like(k), dv=f32(v))   # mixed gradient types
    with pytest.raises(ValueError):
        binding.varlen_attn_bwd(do, q, k, v, o, lse, seg, workspace=torch.empty(64 * 4, dtype=torch.float16, device=DEV))
    with pytest.raises(ValueError):
        binding.varlen_attn_bwd(do, q, k, v, o, lse, seg, workspace=torch.empty(10, dtype=torch.float32, device=DEV))
    with pytest.raises(ValueError):
        binding.varlen_attn_bwd(do, q, k, v, o, lse, seg, dq=torch.empty(q.shape, dtype=torch.float32))   # host tensor
    dq, dk, dv = binding.varlen_attn_bwd(do, q, k, v, o, lse, seg, dq=f32(q), dk=f32(k), dv=f32(v))   # fp32 grads by example
    assert dq.dtype == torch.float32 and bool(torch.isfinite(dk).all())


def test_cross_example_tiles_are_skipped():
    # The schedule visits only key tiles that intersect an example's causal triangle.  Output parity cannot
    # tell a skipped tile from a computed-and-masked one; time can: the same rows take several times longer
    # when their ids never restart (one example per row: every tile below the diagonal is live).  With
    # examples of 8..128 tokens in rows of 8192 the live pairs differ by 90x; the kernels are then bound by
    # bytes, so the measured ratio is smaller (11x on the benchmark's config 4), but far above the 3x asked here.
    rng = np.random.default_rng(8)
    T, R, H, d = 8192, 2, 8, 128
    rows = []
    for _ in range(R):
        row, left = [], T
        while left > 0:
            L = int(min(left, rng.integers(8, 129)))
            row.append(L)
            left -= L
        rows.append(row)
    g = torch.Generator(device=DEV)
    g.manual_seed(1)
    mk = lambda: torch.randn((R * T, H, d), device=DEV, generator=g, dtype=torch.float32).to(torch.bfloat16)
    q, k, v, do = mk(), mk(), mk(), mk()

    def step_ms(pos_np):
        seg = binding.pack_to_cu_seqlens(torch.from_numpy(pos_np).to(DEV))
        o, lse = binding.varlen_attn_fwd(q, k, v, seg)
        ws, dq, dk, dv = binding.bwd_workspace(q, k), torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
        run = lambda: (binding.varlen_attn_fwd(q, k, v, seg, out=o, lse=lse),
                       binding.varlen_attn_bwd(do, q, k, v, o, lse, seg, dq=dq, dk=dk, dv=dv, workspace=ws))
        for _ in range(3):
            run()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(10):
            run()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / 10

    packed = step_ms(wl.position_ids_from_lengths(rows))
    unbroken = step_ms(np.tile(np.arange(T, dtype=np.int64), (R, 1)))
    print(f"   packed {packed:.3f} ms, ids that never restart {unbroken:.3f} ms, ratio {unbroken / packed:.1f}", flush=True)
    assert unbroken > 3.0 * packed


def test_plan_buffer_is_not_overrun():
    # the scan writes cu_seqlens, per-token arrays, tile orders and its scratch inside va_plan_bytes
    for R, T in ((1, 16), (3, 319), (1, 8192), (2, 9000), (5, 20000)):
        nbytes = binding.lib().va_plan_bytes(R, T)
        (plan,), check = _guarded([((nbytes // 4,), torch.int32)])
        seg = binding.Segments.__new__(binding.Segments)
        seg.rows, seg.tokens_per_row, seg.n_tokens, seg.plan, seg.c = R, T, R * T, plan, binding.VaSegments()
        import ctypes as C
        assert binding.lib().va_segments_bind(plan.data_ptr(), nbytes, R, T, C.byref(seg.c)) == 0
        rng = np.random.default_rng(R * 100000 + T)
        pos = (rng.integers(0, 50, size=(R, T)) != 0).astype(np.int64)   # a zero (= boundary) every ~50 tokens
        binding.pack_to_cu_seqlens(torch.from_numpy(pos).to(DEV), seg)
        check()
        assert_seg_equal(seg.host(), oracle.pack(pos))


def test_standalone_D_kernel_on_16bit_inputs():
    # VA_STAGE_D alone on bf16, d = 128: the 16-lanes-per-row kernel that the full MFMA backward never launches
    N, hq, d = 1000, 3, 128
    rng = np.random.default_rng(5)
    do_np, o_np = (wl.round_to_bf16(rng.standard_normal((N, hq, d), dtype=np.float32)) for _ in range(2))
    do, o = to_dev(do_np, "bf16"), to_dev(o_np, "bf16")
    seg = binding.pack_to_cu_seqlens(torch.arange(N, device=DEV)[None, :])
    k = torch.zeros((N, 1, d), device=DEV, dtype=torch.bfloat16)
    lse = torch.zeros((hq, N), device=DEV, dtype=torch.float32)
    ws = binding.bwd_workspace(do, k)
    ws.fill_(float("nan"))
    binding.varlen_attn_bwd(do, do, k, k, o, lse, seg, workspace=ws, stages=binding.STAGE_D)
    torch.cuda.synchronize()
    got = ws[: hq * N].view(hq, N).cpu().numpy().astype(np.float64)
    want = (do_np.astype(np.float64) * o_np.astype(np.float64)).sum(axis=2).T   # D[h, i] = sum_c dO O
    assert np.isfinite(got).all()
    assert np.abs(got - want).max() <= 1e-4 and rel_l2(got, want) <= 1e-6


def test_plain_kernels_forced_on_an_mfma_shape():
    # VA_FORCE_GENERIC=1 is read when the library is first used, so the case runs in a child process
    code = (
        "import sys, torch\n"
        f"sys.path.insert(0, {ROOT!r})\n"
        "from paper_2407_09105_amd import workloads as wl\n"
        "from tests.gpu_util import assert_close, run_gpu, run_oracle\n"
        "w = wl.make_custom([[100, 219], [319]], 4, 2, 128, 'bf16', seed=91)\n"
        "got, ref = run_gpu(w, grad_dtype=torch.float32, nan_fill=True), run_oracle(w)\n"
        "e = assert_close(got, ref, 'bf16')\n"
        # fp32 arithmetic on bf16 inputs: only the bf16 store of O (and its trace in D) is left
        "assert e['dV'][1] <= 1e-5 and e['O'][1] <= 2e-3 and e['dQ'][1] <= 1.5e-3 and e['dK'][1] <= 1.5e-3, e\n"
        "print('forced-generic ok')\n")
    env = dict(os.environ, VA_FORCE_GENERIC="1")
    p = subprocess.run([sys.executable, "-c", code], env=env, capture_output=True, text=True, timeout=300)
    print(p.stdout, p.stderr[-2000:], flush=True)
    assert p.returncode == 0 and "forced-generic ok" in p.stdout


@pytest.mark.parametrize("packer", ["ffd", "sorted", "random", "stream"])
def test_sampler_packs_through_the_whole_path(packer):
    # One pool of examples (lengths 1 .. 700, a few longer than a row), packed into rows of 512 tokens by
    # each sampler of Table 1: rows with a pad tail (one pad pseudo-example), examples truncated to the
    # row, and - for the stream packer - examples broken at a row end.  pack -> forward -> backward
    # against the oracle, element by element.
    rng = np.random.default_rng(31)
    pool = [int(x) for x in np.concatenate([rng.integers(1, 200, size=40), rng.integers(300, 701, size=6)])]
    T = 512
    rows = pk.PACKERS[packer](pool, T)
    pos = pk.position_ids(rows, T)
    lens = pk.row_lengths(rows, T)
    if packer == "stream":
        assert any(len({i for i, _ in r} & {i for i, _ in rows[n + 1]}) for n, r in enumerate(rows[:-1]))   # a broken example
    else:
        assert any(sum(L for _, L in r) < T for r in rows)                                                  # a pad tail
    w = wl.make_custom(lens, 4, 2, 128, "bf16", seed=300)
    assert np.array_equal(w.position_ids, pos)
    print(f"case: {packer}: {len(rows)} rows of {T}, fill {pk.efficiency(rows, T):.3f}", flush=True)
    got = run_gpu(w, grad_dtype=torch.float32, nan_fill=True)
    ref = run_oracle(w)
    assert_seg_equal(got["seg"], ref["seg"])
    assert_close(got, ref, "bf16")
