"""Helpers of the GPU parity tests: move seeded workloads to the device, run the library through
its C ABI (paper_2407_09105_amd.binding), and compare with the CPU oracle."""
import time

import numpy as np
import torch

from oracle import oracle
from paper_2407_09105_amd import binding
from tests.conftest import progress

DEV = "cuda:0"

# bf16 inputs, fp32 accumulation: the bar set for this build (max-abs 2e-2, relative L2 5e-3);
# fp32 path: relative L2 1e-4.
BF16_MAX_ABS, BF16_REL_L2, F32_REL_L2 = 2e-2, 5e-3, 1e-4


def to_dev(a: np.ndarray, dtype: str) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    if dtype == "bf16":
        return t.to(torch.bfloat16)                            # exact: values are already bf16
    return t.to(torch.float16) if dtype == "f16" else t        # exact likewise


def rel_l2(x: np.ndarray, ref: np.ndarray) -> float:
    den = float(np.sqrt((ref.astype(np.float64) ** 2).sum()))
    num = float(np.sqrt(((x.astype(np.float64) - ref) ** 2).sum()))
    return num / den if den > 0 else num


def max_abs(x, ref) -> float:
    return float(np.abs(x.astype(np.float64) - ref).max()) if x.size else 0.0


def bench_hint(w):
    """The example-length hint bench.py passes for this workload (same rule: mean length against 1024)."""
    n = int(oracle.pack(w.position_ids)["cu_seqlens"].size) - 1
    return binding.HINT_LONG_EXAMPLES if w.position_ids.size >= 1024 * n else binding.HINT_SHORT_EXAMPLES


def run_gpu(w, grad_dtype=None, scale=0.0, pos_dtype=torch.int64, nan_fill=False, hint=0):
    """Full path on the GPU: pack -> fwd -> bwd.  Returns host numpy arrays (float64).
    nan_fill: the outputs start as NaN, so that an element no workgroup writes shows.
    hint: an example-length hint for the backward (0: the device chooses the dK/dV shape)."""
    dt = w.cfg.dtype
    pos = torch.from_numpy(w.position_ids).to(DEV).to(pos_dtype)
    q, k, v, do = (to_dev(a, dt) for a in (w.q, w.k, w.v, w.do))
    seg = binding.pack_to_cu_seqlens(pos)
    pre = {}
    if nan_fill:
        gdt = q.dtype if grad_dtype is None else grad_dtype
        nan = lambda shape, dtype: torch.full(shape, float("nan"), dtype=dtype, device=DEV)
        pre = dict(out=nan(q.shape, q.dtype), lse=nan((q.shape[1], q.shape[0]), torch.float32),
                   dq=nan(q.shape, gdt), dk=nan(k.shape, gdt), dv=nan(v.shape, gdt))
    o, lse = binding.varlen_attn_fwd(q, k, v, seg, scale, out=pre.get("out"), lse=pre.get("lse"))
    stages = (binding.STAGE_D | binding.STAGE_DQ | binding.STAGE_DKDV | hint) if hint else None
    dq, dk, dv = binding.varlen_attn_bwd(do, q, k, v, o, lse, seg, scale, grad_dtype=grad_dtype,
                                         dq=pre.get("dq"), dk=pre.get("dk"), dv=pre.get("dv"), stages=stages)
    torch.cuda.synchronize()
    f = lambda t: t.float().cpu().numpy().astype(np.float64)
    return {"seg": seg.host(), "O": f(o), "LSE": f(lse), "dQ": f(dq), "dK": f(dk), "dV": f(dv)}


def run_oracle(w, scale=None):
    seg = oracle.pack(w.position_ids)
    O, LSE = oracle.fwd(w.q, w.k, w.v, seg["cu_seqlens"], scale)
    dQ, dK, dV = oracle.bwd(w.do, w.q, w.k, w.v, seg["cu_seqlens"], scale)
    return {"seg": seg, "O": O, "LSE": LSE, "dQ": dQ, "dK": dK, "dV": dV}


def run_oracle_in_steps(w, long_pairs=4_000_000, heads_per_call=16):
    """The same results as run_oracle for the large configurations, in several oracle calls with a
    progress line after each (one call on config 5 is minutes of silent CPU work).  Examples are
    independent, and so are KV-head groups, so the stream is split without touching the arithmetic:
      - all examples of fewer than `long_pairs` pairs: ONE call on the stream they form when
        concatenated, with the real head layout;
      - each longer example: calls of `heads_per_call` query heads, every query head with its own copy
        of its KV head (grouped-query attention on repeated KV heads is multi-head attention: one of
        the oracle's CPU pins), dK / dV then summed over the heads of a group.  The oracle threads
        over (example, KV head), so this keeps all cores busy on a single example.
    """
    seg = oracle.pack(w.position_ids)
    cu = seg["cu_seqlens"].astype(np.int64)
    N, hq, d = w.q.shape
    hkv = w.k.shape[1]
    G = hq // hkv
    O = np.zeros((N, hq, d)); dQ = np.zeros((N, hq, d)); LSE = np.zeros((hq, N))
    dK = np.zeros((N, hkv, d)); dV = np.zeros((N, hkv, d))
    L = np.diff(cu)
    pairs = L * (L + 1) // 2
    t0 = time.time()
    short = np.flatnonzero(pairs < long_pairs)
    if short.size:
        idx = np.concatenate([np.arange(cu[s], cu[s + 1]) for s in short])
        cu_s = np.concatenate([[0], np.cumsum(L[short])]).astype(np.int32)
        q, k, v, do = w.q[idx], w.k[idx], w.v[idx], w.do[idx]
        O[idx], lse = oracle.fwd(q, k, v, cu_s)
        LSE[:, idx] = lse
        dQ[idx], dK[idx], dV[idx] = oracle.bwd(do, q, k, v, cu_s)
        progress(f"   oracle: {short.size} examples of fewer than {long_pairs} pairs done, {time.time() - t0:.0f} s")
    for s in np.flatnonzero(pairs >= long_pairs):
        a, b = int(cu[s]), int(cu[s + 1])
        cu_1 = np.array([0, b - a], dtype=np.int32)
        for h0 in range(0, hq, heads_per_call):
            hs = np.arange(h0, min(h0 + heads_per_call, hq))
            q, do = w.q[a:b, hs], w.do[a:b, hs]
            k, v = w.k[a:b, hs // G], w.v[a:b, hs // G]          # one KV copy per query head
            O[a:b, hs], lse = oracle.fwd(q, k, v, cu_1)
            LSE[hs, a:b] = lse
            dq, dk, dv = oracle.bwd(do, q, k, v, cu_1)
            dQ[a:b, hs] = dq
            np.add.at(dK[a:b], (slice(None), hs // G), dk)
            np.add.at(dV[a:b], (slice(None), hs // G), dv)
            progress(f"   oracle: example of {b - a} tokens, query heads {h0}..{hs[-1]} done, {time.time() - t0:.0f} s")
    return {"seg": seg, "O": O, "LSE": LSE, "dQ": dQ, "dK": dK, "dV": dV}


def assert_seg_equal(got: dict, ref: dict):
    assert got["n"] == ref["n"]
    assert got["max_seqlen"] == ref["max_seqlen"]
    for key in ("cu_seqlens", "seg_id", "seg_start", "seg_end"):
        assert got[key].dtype == np.int32
        assert np.array_equal(got[key], ref[key]), key


def assert_close(got: dict, ref: dict, dtype: str, what=("O", "dQ", "dK", "dV"), bf16_stored=()):
    """bf16 bar: max-abs <= 2e-2 and rel-L2 <= 5e-3 for O (always stored in the input dtype) and
    for gradients emitted in fp32.  A gradient that is *stored* in bf16 carries, on top of the arithmetic error, the rounding of
    the store itself (half an ulp = 2^-9 |x|, which exceeds 2e-2 once |x| > 5.1, as summed GQA
    gradients do); for those the element-wise bound is 2e-2 + 2^-8 |ref| (rel-L2 unchanged)."""
    errs = {}
    for key in what:
        errs[key] = (max_abs(got[key], ref[key]), rel_l2(got[key], ref[key]))
    errs["LSE"] = (max_abs(got["LSE"], ref["LSE"]), 0.0)
    print("   errors (max-abs, rel-L2):", {k: (f"{a:.2e}", f"{b:.2e}") for k, (a, b) in errs.items()}, flush=True)
    for key in what:
        ma, rl = errs[key]
        if dtype in ("bf16", "f16"):   # the 16-bit paths share the bar (fp16 rounds P and dS finer than bf16)
            assert rl <= BF16_REL_L2, (key, errs)
            if key in bf16_stored:
                excess = np.abs(got[key] - ref[key]) - (BF16_MAX_ABS + np.abs(ref[key]) / 256.0)
                assert excess.max() <= 0, (key, errs)
            else:
                assert ma <= BF16_MAX_ABS, (key, errs)
        else:
            assert rl <= F32_REL_L2, (key, errs)
    assert errs["LSE"][0] <= (1e-3 if dtype in ("bf16", "f16") else 1e-5), errs
    return errs
