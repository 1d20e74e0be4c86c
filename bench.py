#!/usr/bin/env python3
"""Benchmark of the packed variable-length attention hot path on one MI355X.

One "step" = one pass of the whole path over one packed batch resident in HBM:
position_ids -> cu_seqlens / tile schedule, forward (O, LSE), backward (dQ, dK, dV).

Prints ONE JSON line.  Its headline (`value`, `roofline`, `cpu_baseline`) is the largest
single-GPU workload, configs[4] (2 x 16384 tokens, 40 / 8 heads, long-tail lengths): useful
(mask-respecting, padding-free) attention TFLOP/s of fwd+bwd, tokens/s, the roofline fraction
of the dominant kernel and the CPU oracle timed on a bounded sample of the same workload.
`per_config` carries the same figures for every bf16 workload (configs[1..4]), each with the
same kernels on the equivalent padded batches and without position ids.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 5] [--only] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_MFMA_TFLOPS = 2500.0   # MI355X dense bf16 matrix peak (published)
PEAK_HBM_GBS = 8000.0            # MI355X HBM3E peak (published)


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=5, help="headline workload (index into the config table, 2..5)")
    ap.add_argument("--only", action="store_true", help="measure the headline workload only (no per_config list)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-padded", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="only the timed step: skip measured peaks, cold-cache, no-position-id, collator and rotary timings")
    ap.add_argument("--no-packers", action="store_true",
                    help="skip the step on packs made by the paper's samplers from one example pool")
    return ap.parse_args()


def flops(cfg, pairs):
    """Useful FLOPs: 4d per unmasked (i, j) pair per query head forward, 10d backward."""
    f = 4 * cfg.d * cfg.hq * pairs
    b = 10 * cfg.d * cfg.hq * pairs
    return f, b


class GpuRun:
    """Device buffers + one `step()` of the path; stage events for per-kernel timing."""

    def __init__(self, torch, binding, pos_np, q, k, v, do, n_examples=None):
        self.torch, self.b = torch, binding
        # the host made these lengths, so it can name the dK/dV kernel's shape instead of having the
        # device pick between two launches (the device's own rule: mean example length >= 1024 tokens)
        self.hint = 0
        if n_examples:
            self.hint = binding.HINT_LONG_EXAMPLES if pos_np.size >= 1024 * n_examples else binding.HINT_SHORT_EXAMPLES
        self.pos = torch.from_numpy(pos_np).cuda()
        self.q, self.k, self.v, self.do = q, k, v, do
        self.seg = binding.Segments(pos_np.shape[0], pos_np.shape[1], "cuda")
        self.o = torch.empty_like(q)
        self.lse = torch.empty((q.shape[1], q.shape[0]), dtype=torch.float32, device="cuda")
        self.dq, self.dk, self.dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
        self.ws = binding.bwd_workspace(q, k)

    def step(self, ev=None):
        b = self.b
        if ev: ev[0].record()
        b.pack_to_cu_seqlens(self.pos, self.seg)
        if ev: ev[1].record()
        b.varlen_attn_fwd(self.q, self.k, self.v, self.seg, out=self.o, lse=self.lse)
        if ev: ev[2].record()
        if ev:
            for i, stage in enumerate((b.STAGE_DQ, b.STAGE_DKDV)):   # the order of the full backward
                b.varlen_attn_bwd(self.do, self.q, self.k, self.v, self.o, self.lse, self.seg, dq=self.dq,
                                  dk=self.dk, dv=self.dv, workspace=self.ws, stages=stage | self.hint)
                ev[3 + i].record()
        else:
            b.varlen_attn_bwd(self.do, self.q, self.k, self.v, self.o, self.lse, self.seg, dq=self.dq,
                              dk=self.dk, dv=self.dv, workspace=self.ws,
                              stages=(b.STAGE_D | b.STAGE_DQ | b.STAGE_DKDV | self.hint) if self.hint else None)


def timed(torch, run, steps, warmup, with_events=True):
    """W warm-up steps, then exactly K timed steps between device synchronisations.
    Returns (ms_per_step, {stage: avg ms}) -- stage times from events recorded inside the timed steps
    on the stream the kernels are launched on (torch's current stream, whose handle the binding passes)."""
    for _ in range(warmup):
        run.step()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(steps)] if with_events else None
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(steps):
        run.step(evs[s] if evs else None)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    stages = {}
    if evs:
        names = ["pack", "fwd", "bwd_dQ", "bwd_dKdV"]   # the dQ kernel also forms D = rowsum(dO * O)
        for i, n in enumerate(names):
            stages[n] = float(np.mean([e[i].elapsed_time(e[i + 1]) for e in evs]))
    return ms, stages


def padded_run(torch, binding, wl, w, q, k, v, do, mode="group_max"):
    """Batch-level padding of the same examples: groups of 4, each right-padded to the group's
    longest (a (4, L_max) batch per group), or - mode "global_max" - every example padded to the
    longest of the workload (the (bs, msl) form); run as examples of uniform length through the same
    kernels.  Pad tokens hold zeros.  Useful FLOPs and tokens counted are the real ones."""
    lay = wl.padded_layout(w.lengths, group=4, mode=mode)
    n_pad = sum(p for _, p in lay)
    pos = np.concatenate([np.arange(p, dtype=np.int64) for _, p in lay])[None, :]
    src = np.concatenate([np.arange(L, dtype=np.int64) for L, _ in lay])            # offsets inside example
    starts_real = np.cumsum([0] + [L for L, _ in lay])[:-1]
    starts_pad = np.cumsum([0] + [p for _, p in lay])[:-1]
    idx_real = np.concatenate([s + np.arange(L) for s, (L, _) in zip(starts_real, lay)])
    idx_pad = np.concatenate([s + np.arange(L) for s, (L, _) in zip(starts_pad, lay)])
    del src
    ir = torch.from_numpy(idx_real).cuda()
    ip = torch.from_numpy(idx_pad).cuda()

    def pad(t):
        out = torch.zeros((n_pad,) + tuple(t.shape[1:]), dtype=t.dtype, device="cuda")
        out[ip] = t[ir]
        return out

    run = GpuRun(torch, binding, pos, pad(q), pad(k), pad(v), pad(do), n_examples=len(lay))
    return run, n_pad, ir, ip


def no_posid_run(torch, binding, w, q, k, v, do):
    """The same packed rows with position ids that never restart (0..T-1 per row): what fixed-length
    packing without position ids computes (Table 1: cross-contaminated attention).  One example per
    row, so no key tile is skipped; useful FLOPs counted are still those of the real examples."""
    cfg = w.cfg
    pos = np.tile(np.arange(cfg.tokens_per_row, dtype=np.int64), (cfg.rows, 1))
    return GpuRun(torch, binding, pos, q, k, v, do, n_examples=cfg.rows)


def collate_timing(torch, binding, w, steps):
    """Device collator (padded batch -> input_ids, labels, position_ids) on the workload's first row."""
    lengths = np.array(w.lengths[0], dtype=np.int32)
    n, Lp, T = len(lengths), int(lengths.max()), w.cfg.tokens_per_row
    g = torch.Generator(device="cuda"); g.manual_seed(7)
    ids = torch.randint(0, 32000, (n, Lp), device="cuda", generator=g, dtype=torch.int64)
    ln = torch.from_numpy(lengths).cuda()
    out = binding.collate_padding_free(ids, ln, T)
    for _ in range(3):
        binding.collate_padding_free(ids, ln, T, out=out)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(steps):
        binding.collate_padding_free(ids, ln, T, out=out)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    algo_bytes = T * 8 + n * 4 + 3 * T * 8 + (n + 1) * 4   # ids read once, lengths, three outputs, offsets
    ok = bool((out["position_ids"].cpu().numpy() == w.position_ids[:1]).all())
    return {"ms": ms, "examples": n, "padded_len": Lp, "tokens": T, "algorithmic_bytes": algo_bytes,
            "achieved_GBs": algo_bytes / (ms * 1e-3) / 1e9, "frac_hbm_peak": algo_bytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
            "bound": "launch latency (two tiny kernels)", "position_ids_match_workload": ok}


def rope_timing(torch, binding, w, q, steps):
    """Rotary embedding of Q in place from the workload's position ids: HBM-bound, one read + one write."""
    pos = torch.from_numpy(w.position_ids).cuda().reshape(-1)
    x = q.clone()
    for _ in range(3):
        binding.rope_apply(x, pos, out=x)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(steps):
        binding.rope_apply(x, pos, out=x)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    algo_bytes = 2 * x.numel() * x.element_size() + pos.numel() * 8
    return {"tensor": "Q " + "x".join(str(s) for s in x.shape) + " bf16, in place", "ms": ms,
            "algorithmic_bytes": algo_bytes, "achieved_GBs": algo_bytes / (ms * 1e-3) / 1e9,
            "frac_hbm_peak": algo_bytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, "bound": "hbm"}


def measured_peaks(torch):
    """What this GPU sustains: a matrix-instruction-only loop and a plain 256 MiB device copy."""
    from paper_2407_09105_amd import probes as binding
    sink = torch.zeros(64, dtype=torch.float32, device="cuda")
    binding.probe_mfma(sink, 2000)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    fl = binding.probe_mfma(sink, 20000)
    e1.record()
    torch.cuda.synchronize()
    mfma = fl / (e0.elapsed_time(e1) * 1e-3) / 1e12
    src = torch.empty(64 * 1024 * 1024, dtype=torch.float32, device="cuda").fill_(1.0)
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(5):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    copy = 5 * 2 * src.numel() * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    # the matrix instructions with realistic operands and in the company they keep in the kernels
    ops = torch.randn(32768, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    clocks = torch.zeros(2, dtype=torch.int64, device="cuda")
    mixes = {}
    for name, lds, valu in (("mfma_only", 0, 0), ("lds16", 16, 0), ("lds8", 8, 0),
                            ("lds16_valu24_fwd_mix", 16, 24), ("lds16_valu12", 16, 12), ("lds8_valu16", 8, 16)):
        for _ in range(12):   # long enough for the clock governor to settle
            fl = binding.probe_mix(ops, lds, valu, sink, clocks, 6000)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(8):
            binding.probe_mix(ops, lds, valu, sink, clocks, 6000)
        e1.record()
        torch.cuda.synchronize()
        c = clocks.cpu().numpy()
        mixes[name] = {"TFLOPs": 8 * fl / (e0.elapsed_time(e1) * 1e-3) / 1e12,
                       "shader_clock_MHz": float(c[0]) / max(float(c[1]), 1.0) * 100.0}
    return {"mfma_bf16_TFLOPs": mfma, "device_copy_GBs": copy,
            "mfma_bf16_mix_TFLOPs": mixes,
            "note": "mfma_bf16_TFLOPs: bf16 32x32x16 matrix instructions only, constant small operands, 2 waves per SIMD; "
                    "mfma_bf16_mix_TFLOPs: the same with N(0,1) bf16 operands plus, per 16 matrix instructions, "
                    "ldsN = N 1 KB fragment reads from LDS and valuM = M groups of {fma, exp2, max, add}, all independent "
                    "(what the power limit and the issue slots leave to the matrix pipe; shader clock read in-kernel); "
                    "device_copy_GBs: 256 MiB device-to-device copy (read + write bytes)"}


def cold_cache_ms(torch, binding, w, q, k, v, do, steps, copies=3):
    """The same step cycling through `copies` independent sets of inputs and outputs (each ~0.5 GB on
    config 2), so that no step finds its tensors in the 256 MB last-level cache."""
    runs = [GpuRun(torch, binding, w.position_ids, q.clone(), k.clone(), v.clone(), do.clone(),
                   n_examples=w.stats["n_segments"]) for _ in range(copies)]
    for r in runs:
        r.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(steps):
        runs[s % copies].step()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def packer_runs(torch, binding, wl, cfg, seed, steps):
    """One pool of examples drawn from the workload's length law (about 4x the workload's tokens),
    packed into rows of the workload's row length by each sampler of Table 1; the same step on each
    pack.  Useful FLOPs and tokens count the real examples only (a row's unused tail is one pad
    pseudo-example: executed, not counted)."""
    from paper_2407_09105_amd import packers as pk
    rng = np.random.default_rng(seed + 7)
    T = cfg.tokens_per_row
    pool, tokens = [], 0
    while tokens < 4 * cfg.n_tokens:
        L = min(wl._draw_len(cfg, rng), T)
        pool.append(L)
        tokens += L
    out = {"pool": {"examples": len(pool), "tokens": tokens, "row_tokens": T}}
    g = torch.Generator(device="cuda"); g.manual_seed(11)
    for name, fn in pk.PACKERS.items():
        rows = fn(pool, T)
        pos = pk.position_ids(rows, T)
        N = pos.size
        mk = lambda h: torch.randn((N, h, cfg.d), device="cuda", generator=g, dtype=torch.float32).to(torch.bfloat16)
        run = GpuRun(torch, binding, pos, mk(cfg.hq), mk(cfg.hkv), mk(cfg.hkv), mk(cfg.hq),
                     n_examples=sum(len(r) for r in rows))
        ms, _ = timed(torch, run, steps, 3, with_events=False)
        pairs = sum(L * (L + 1) // 2 for r in rows for _, L in r)
        fl = sum(flops(cfg, pairs))
        out[name] = {"rows": len(rows), "fill": pk.efficiency(rows, T), "ms_per_step": ms,
                     "value": fl / (ms * 1e-3) / 1e12, "unit": "TFLOP/s (useful)",
                     "tokens_per_s": sum(L for r in rows for _, L in r) / (ms * 1e-3)}
        del run
    return out


# The CPU-oracle sample of each workload: (query heads, KV heads, longest example kept).  Configs 2-4 run
# in full.  Config 5 is 6 TFLOP of fp64 work (minutes); the oracle threads over (example, KV head), so
# its three longest examples (8708, 5965, 5647 tokens: tasks of up to 100 s each) are left out and the
# other 21 run with every head, which keeps the cores busy; the rate is what is reported, the time of
# the whole workload is extrapolated from it.
CPU_SAMPLE = {2: (32, 32, None), 3: (32, 8, None), 4: (32, 32, None), 5: (40, 8, 4400)}


def cpu_baseline(wl, cfg_id):
    """The oracle as it stands, timed on the host cores, on a bounded sample of the workload: the
    same packed examples (all, or those up to a length cap) with all or some KV-head groups (work is
    exactly linear in groups).  `value` is the oracle's rate on the sample's own useful FLOPs."""
    from oracle import oracle
    cfg = wl.CONFIGS[cfg_id]
    hq_s, hkv_s, cap = CPU_SAMPLE[cfg_id]
    w = wl.make_workload(cfg_id, hq=hq_s, hkv=hkv_s)
    cu = oracle.pack(w.position_ids)["cu_seqlens"].astype(np.int64)
    L = np.diff(cu)
    keep = np.arange(L.size) if cap is None else np.flatnonzero(L <= cap)
    idx = np.concatenate([np.arange(cu[s], cu[s + 1]) for s in keep])
    cu_s = np.concatenate([[0], np.cumsum(L[keep])]).astype(np.int32)
    q, k, v, do = w.q[idx], w.k[idx], w.v[idx], w.do[idx]
    t0 = time.perf_counter()
    oracle.fwd(q, k, v, cu_s)
    oracle.bwd(do, q, k, v, cu_s)
    dt = time.perf_counter() - t0
    pairs = int((L[keep] * (L[keep] + 1) // 2).sum())
    f, b = flops(w.cfg, pairs)
    rate = (f + b) / dt
    full = sum(flops(cfg, w.stats["pairs"]))
    whole = cap is None and hq_s == cfg.hq
    return {
        "value": rate / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
        "sample": (f"the whole workload, fwd+bwd in fp64, {dt:.1f} s" if whole else
                   f"{hq_s} of {cfg.hq} query heads ({hkv_s} of {cfg.hkv} KV groups) and the {keep.size} of {L.size} "
                   f"examples of at most {cap} tokens ({pairs} of {w.stats['pairs']} pairs per head) of the same "
                   f"packed batch, fwd+bwd in fp64, {dt:.1f} s; the whole workload extrapolated x{full / (f + b):.1f}"),
        "seconds": dt, "full_workload_seconds": dt if whole else full / rate,
        "full_workload_seconds_is": "measured" if whole else "extrapolated from the sample's rate",
        "tokens_per_s_equiv": cfg.n_tokens / (full / rate),
    }


def read_traffic(cfg_id, kernel):
    """HBM bytes per launch from the committed rocprofv3 counter summary, if there is one."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_cfg{cfg_id}.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        parts = line.split()
        if len(parts) >= 2 and parts[0] == kernel + ":":
            try:
                return float(parts[1])
            except ValueError:
                return None
    return None


KERNEL_NAMES = {"fwd": "fwd_mfma_kernel", "bwd_dKdV": "dkdv_mfma_kernel", "bwd_dQ": "dq_mfma_kernel"}


def algorithmic_work(cfg, pairs, e=2, eg=2):
    """Per launch and kernel: (algorithmic FLOPs, algorithmic HBM bytes).
    FLOPs per unmasked pair per query head: forward 4d; the backward's 10d split as 8d to the dK/dV
    kernel (S, dP, dV, dK) and 2d to the dQ kernel (dQ; its own recomputation of S and dP is overhead,
    not algorithmic work).  Bytes: every operand and result of the kernel once (e bytes per input
    element, eg per gradient element, 4 per row statistic)."""
    n, d, hq, hkv = cfg.n_tokens, cfg.d, cfg.hq, cfg.hkv
    ph = pairs * hq
    return {
        # reads Q, K, V; writes O and the row log-sum-exp
        "fwd": (4 * d * ph, n * (e * d * (2 * hq + 2 * hkv) + 4 * hq)),
        # reads Q, dO, K, V, LSE, D; writes dK, dV
        "bwd_dKdV": (8 * d * ph, n * (e * d * (2 * hq + 2 * hkv) + eg * d * 2 * hkv + 8 * hq)),
        # reads Q, dO, O, K, V, LSE; writes dQ and D
        "bwd_dQ": (2 * d * ph, n * (e * d * (3 * hq + 2 * hkv) + eg * d * hq + 8 * hq)),
    }


def roofline_of(cfg, pairs, stages, cfg_id):
    """Roofline object of the kernel with the longest average launch.  The bound is the one the
    kernel's algorithmic intensity selects: below the ridge (bf16 MFMA peak / HBM peak, in FLOP per
    byte) the launch cannot beat the time its algorithmic bytes take, above it the time of its FLOPs."""
    work = algorithmic_work(cfg, pairs)
    dom = max(work, key=lambda s: stages[s])
    fl, by = work[dom]
    sec = stages[dom] * 1e-3
    ridge = PEAK_BF16_MFMA_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9)
    if fl / by >= ridge:
        bound, achieved, peak, unit = "mfma", fl / sec / 1e12, PEAK_BF16_MFMA_TFLOPS, "TFLOP/s"
    else:
        bound, achieved, peak, unit = "hbm", by / sec / 1e9, PEAK_HBM_GBS, "GB/s"
    return {
        "kernel": KERNEL_NAMES[dom], "bound": bound, "achieved": achieved, "peak": peak, "unit": unit,
        "frac": achieved / peak, "traffic": read_traffic(cfg_id, KERNEL_NAMES[dom]),
        "traffic_source": f"profiles/hbm_traffic_cfg{cfg_id}.txt (FETCH_SIZE + WRITE_SIZE of separate rocprofv3 --pmc "
                          "runs of this command, per launch; read from that file, not measured in this run)",
        "avg_kernel_ms": stages[dom],
        "avg_kernel_ms_is": "HIP-event interval around this kernel's launch alone (its one working shape), on the "
                            "launch stream, averaged over the timed steps",
        "algorithmic_flops": fl, "algorithmic_bytes": by, "flop_per_byte": fl / by, "ridge_flop_per_byte": ridge,
        "all_kernels": {KERNEL_NAMES[s]: {"ms": stages[s],
                                          "algorithmic_TFLOPs": work[s][0] / (stages[s] * 1e-3) / 1e12,
                                          "frac_of_bf16_mfma_peak": work[s][0] / (stages[s] * 1e-3) / 1e12 / PEAK_BF16_MFMA_TFLOPS,
                                          "algorithmic_GBs": work[s][1] / (stages[s] * 1e-3) / 1e9,
                                          "frac_of_hbm_peak": work[s][1] / (stages[s] * 1e-3) / 1e9 / PEAK_HBM_GBS,
                                          "flop_per_byte": work[s][0] / work[s][1]}
                        for s in work},
    }


def bench_config(torch, binding, wl, cfg_id, args, headline):
    """Everything measured on one workload -> dict (the per_config entry)."""
    w = wl.make_workload(cfg_id)
    cfg = w.cfg
    assert cfg.dtype == "bf16"
    to_dev = lambda a: torch.from_numpy(a).cuda().to(torch.bfloat16)
    q, k, v, do = to_dev(w.q), to_dev(w.k), to_dev(w.v), to_dev(w.do)
    run = GpuRun(torch, binding, w.position_ids, q, k, v, do, n_examples=w.stats["n_segments"])
    ms, stages = timed(torch, run, args.steps, args.warmup)
    # the same K steps without stage events (the figure reported as `value`)
    ms_plain, _ = timed(torch, run, args.steps, 2, with_events=False)
    f_fwd, f_bwd = flops(cfg, w.stats["pairs"])
    useful = f_fwd + f_bwd
    value = useful / (ms_plain * 1e-3) / 1e12
    # minimum HBM traffic of the whole step (each tensor once) -> fraction of the HBM roofline
    e = 2
    hbm_min = cfg.n_tokens * (6 * e * cfg.d * (cfg.hq + cfg.hkv) + 12 * cfg.hq)
    out = {
        "config": {"workload": f"configs[{cfg_id - 1}] {cfg.name}: {cfg.rows} packed row(s) x {cfg.tokens_per_row} tokens, "
                               f"Hq={cfg.hq} Hkv={cfg.hkv} d={cfg.d}, seed {w.seed}",
                   "n_tokens": cfg.n_tokens, "n_examples": w.stats["n_segments"], "len_min": w.stats["len_min"],
                   "len_median": w.stats["len_median"], "len_max": w.stats["len_max"], "pairs_per_head": w.stats["pairs"],
                   "grad_dtype": "bf16",
                   "dkdv_shape_hint": {0: "none", binding.HINT_LONG_EXAMPLES: "long examples", binding.HINT_SHORT_EXAMPLES: "short examples"}[run.hint]},
        "value": value, "unit": "TFLOP/s", "ms_per_step": ms_plain, "tokens_per_s": cfg.n_tokens / (ms_plain * 1e-3),
        "frac_bf16_mfma_peak": value / PEAK_BF16_MFMA_TFLOPS,
        "frac_hbm_peak_at_min_traffic": hbm_min / (ms_plain * 1e-3) / 1e9 / PEAK_HBM_GBS,
        "stage_ms": stages, "ms_per_step_with_stage_events": ms,
        "useful_gflop": {"fwd": f_fwd / 1e9, "bwd": f_bwd / 1e9},
        "roofline": roofline_of(cfg, w.stats["pairs"], stages, cfg_id),
    }
    k_steps = max(5, args.steps // 2)
    if not args.no_padded:
        out["padded"] = {}
        for mode, what in (("group_max", "groups of 4 examples, each right-padded to the group's longest (batch-level padding)"),
                           ("global_max", "every example right-padded to the longest of the workload")):
            prun, n_pad, _, _ = padded_run(torch, binding, wl, w, q, k, v, do, mode=mode)
            pms, _ = timed(torch, prun, k_steps, 3, with_events=False)
            out["padded"][mode] = {
                "layout": what, "padded_tokens": n_pad, "ms_per_step": pms, "value": useful / (pms * 1e-3) / 1e12,
                "unit": "TFLOP/s (useful)", "tokens_per_s": cfg.n_tokens / (pms * 1e-3), "packing_gain": pms / ms_plain,
            }
            del prun
            torch.cuda.empty_cache()
    if not args.no_extras:
        nrun = no_posid_run(torch, binding, w, q, k, v, do)
        nms, _ = timed(torch, nrun, k_steps, 3, with_events=False)
        del nrun
        T = cfg.tokens_per_row
        out["no_position_ids"] = {
            "layout": "same rows, ids 0..T-1 (one example per row: attention crosses example boundaries)",
            "ms_per_step": nms, "value": useful / (nms * 1e-3) / 1e12, "unit": "TFLOP/s (useful)",
            "executed_pairs_per_head": cfg.rows * T * (T + 1) // 2, "position_id_gain": nms / ms_plain,
        }
        if headline:
            cold = cold_cache_ms(torch, binding, w, q, k, v, do, args.steps)
            out["cold_cache"] = {"ms_per_step": cold, "value": useful / (cold * 1e-3) / 1e12, "unit": "TFLOP/s (useful)",
                                 "note": "3 input/output sets cycled; `value` above re-uses one set (inputs partly cache-resident)"}
            out["collate"] = collate_timing(torch, binding, w, args.steps)
            out["rope"] = rope_timing(torch, binding, w, q, args.steps)
    if headline and not args.no_packers:
        out["packers"] = packer_runs(torch, binding, wl, cfg, w.seed, max(5, args.steps // 4))
    del run, q, k, v, do
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, cfg_id)
    return out


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (one process, no collectives); "
              f"--gpus {args.gpus} is not supported. Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2407_09105_amd import binding, workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    binding.lib()  # fail loudly if the HIP library is not built

    # one plain device-to-device copy of known size (256 MiB read + 256 MiB written), outside every
    # timed region: under `rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE` it calibrates the counters' units
    calib_src = torch.empty(64 * 1024 * 1024, dtype=torch.float32, device="cuda").fill_(1.0)
    calib_dst = torch.empty_like(calib_src)
    calib_dst.copy_(calib_src)
    torch.cuda.synchronize()
    del calib_src, calib_dst

    cfg_ids = [args.config] if args.only else sorted({2, 3, 4, 5} | {args.config}, key=lambda c: (c == args.config, c))
    per_config = []
    for c in cfg_ids:
        print(f"bench.py: config {c} ...", file=sys.stderr, flush=True)
        per_config.append(bench_config(torch, binding, wl, c, args, headline=(c == args.config)))
    head = per_config[-1]
    out = {
        "metric": "useful attention TFLOP/s (fwd+bwd), packed, one GPU",
        "value": head["value"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
    }
    out.update({k: v for k, v in head.items() if k not in out})
    if not args.no_extras:
        out["measured_peaks"] = measured_peaks(torch)
        out["frac_measured_mfma_peak"] = head["value"] / out["measured_peaks"]["mfma_bf16_TFLOPs"]
    if "cpu_baseline" not in out:
        out["cpu_baseline"] = None
    out["per_config"] = sorted(per_config, key=lambda r: r["config"]["workload"])
    print(json.dumps(out))


if __name__ == "__main__":
    main()
