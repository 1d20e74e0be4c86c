"""Seeded synthetic workloads for packed variable-length attention.

This module only *draws inputs*: example lengths, the position_ids a
padding-free collator would emit for them (Section 3.1: ids run 0..L-1 per
example and restart at 0), and Gaussian Q/K/V/dO tensors.  It contains none of
the attention arithmetic, so both the CPU oracle's tests and the GPU path's
tests may import it without sharing any of the method's code.

The length laws stand in for the length histograms of the three fine-tuning
datasets the paper measures on (Section 4, Figure 1: one with a mode near 100
tokens, one near 400, one long and high-variance); the row shapes are the
paper's (bs, msl) grid (Section 4.1 and the tables of Section 4.3).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

SEED_BASE = 240709105


@dataclass(frozen=True)
class Config:
    cfg: int
    name: str
    rows: int            # R: packed rows (batch elements)
    tokens_per_row: int  # T
    hq: int
    hkv: int
    d: int
    dtype: str           # "f32" | "bf16"
    law: str             # "fixed" | "lognormal" | "uniform" | "longtail"
    law_args: tuple = ()

    @property
    def n_tokens(self) -> int:
        return self.rows * self.tokens_per_row


CONFIGS = {
    1: Config(1, "tiny-fp32-smoke", 1, 16, 2, 2, 16, "f32", "fixed", ((3, 5, 1, 7),)),
    2: Config(2, "llama2-7b-like-1x8192", 1, 8192, 32, 32, 128, "bf16", "lognormal", (256.0, 1.0, 16, 4096)),
    3: Config(3, "mistral-7b-like-gqa-4x4096", 4, 4096, 32, 8, 128, "bf16", "lognormal", (512.0, 0.8, 32, 4096)),
    4: Config(4, "many-short-8x8192", 8, 8192, 32, 32, 128, "bf16", "uniform", (8, 128)),
    5: Config(5, "long-tail-gqa-2x16384", 2, 16384, 40, 8, 128, "bf16", "longtail", (300.0, 1.2, 0.1, 4096, 16384)),
}


def _lognormal_len(rng, median, sigma, lo, hi):
    z = rng.standard_normal()
    L = int(math.floor(math.exp(math.log(median) + sigma * z) + 0.5))
    return max(lo, min(hi, L))


def _draw_len(cfg: Config, rng) -> int:
    if cfg.law == "lognormal":
        median, sigma, lo, hi = cfg.law_args
        return _lognormal_len(rng, median, sigma, lo, hi)
    if cfg.law == "uniform":
        lo, hi = cfg.law_args
        return int(rng.integers(lo, hi + 1))
    if cfg.law == "longtail":
        median, sigma, p_long, lo_long, hi_long = cfg.law_args
        u = rng.random()
        if u < p_long:
            return int(rng.integers(lo_long, hi_long + 1))
        return _lognormal_len(rng, median, sigma, 1, cfg.tokens_per_row)
    raise ValueError(cfg.law)


def draw_lengths(cfg: Config, rng) -> List[List[int]]:
    """Example lengths per row; each row is filled exactly, the last example of
    a row being cut to what is left (a fixed-length pack may break its last
    example, Table 1)."""
    if cfg.law == "fixed":
        rows = [list(cfg.law_args[0]) for _ in range(cfg.rows)]
        for r in rows:
            assert sum(r) == cfg.tokens_per_row
        return rows
    out = []
    for _ in range(cfg.rows):
        filled, row = 0, []
        while filled < cfg.tokens_per_row:
            L = _draw_len(cfg, rng)
            if filled + L >= cfg.tokens_per_row:
                L = cfg.tokens_per_row - filled
            row.append(L)
            filled += L
        out.append(row)
    return out


def position_ids_from_lengths(lengths_per_row: List[List[int]], dtype=np.int64) -> np.ndarray:
    """[R, T] ids: 0..L-1 for each example, concatenated (Section 3.1)."""
    rows = [np.concatenate([np.arange(L, dtype=dtype) for L in row]) for row in lengths_per_row]
    T = len(rows[0])
    assert all(len(r) == T for r in rows), "rows must have equal token counts"
    return np.stack(rows, axis=0)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); returned as
    float32 holding exactly representable bf16 values."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = (u + bias) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def round_to_f16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest IEEE half (ties to even); returned as float32."""
    return np.ascontiguousarray(x, dtype=np.float32).astype(np.float16).astype(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of float32 values that are exactly bf16."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    return (u >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class Workload:
    cfg: Config
    seed: int
    lengths: List[List[int]]
    position_ids: np.ndarray           # int64 [R, T]
    q: Optional[np.ndarray] = None     # float32 [N, Hq, d]  (bf16-exact when cfg.dtype == "bf16")
    k: Optional[np.ndarray] = None     # float32 [N, Hkv, d]
    v: Optional[np.ndarray] = None
    do: Optional[np.ndarray] = None    # float32 [N, Hq, d]
    stats: dict = field(default_factory=dict)


def length_stats(lengths_per_row: List[List[int]]) -> dict:
    flat = np.array([L for row in lengths_per_row for L in row], dtype=np.int64)
    pairs = int((flat * (flat + 1) // 2).sum())
    return {
        "n_segments": int(flat.size),
        "len_min": int(flat.min()),
        "len_median": float(np.median(flat)),
        "len_max": int(flat.max()),
        "pairs": pairs,                      # unmasked (i, j) pairs per head
        "tokens": int(flat.sum()),
    }


def make_workload(cfg_id: int, seed: Optional[int] = None, tensors: bool = True,
                  hq: Optional[int] = None, hkv: Optional[int] = None) -> Workload:
    """Draw config `cfg_id`.  Lengths first, then Q, K, V, dO ~ N(0,1) in that
    order from the same generator.  `hq`/`hkv` override the head counts (used
    by tests that want the same length mix on fewer heads)."""
    cfg = CONFIGS[cfg_id]
    if hq is not None or hkv is not None:
        cfg = Config(cfg.cfg, cfg.name + "-heads-overridden", cfg.rows, cfg.tokens_per_row,
                     hq or cfg.hq, hkv or cfg.hkv, cfg.d, cfg.dtype, cfg.law, cfg.law_args)
    seed = SEED_BASE + cfg_id if seed is None else seed
    rng = np.random.default_rng(seed)
    lengths = draw_lengths(cfg, rng)
    pos = position_ids_from_lengths(lengths)
    w = Workload(cfg, seed, lengths, pos, stats=length_stats(lengths))
    if tensors:
        N = cfg.n_tokens
        shapes = [(N, cfg.hq, cfg.d), (N, cfg.hkv, cfg.d), (N, cfg.hkv, cfg.d), (N, cfg.hq, cfg.d)]
        arrs = [rng.standard_normal(s, dtype=np.float32) for s in shapes]
        if cfg.dtype == "bf16":
            arrs = [round_to_bf16(a) for a in arrs]
        w.q, w.k, w.v, w.do = arrs
    return w


def make_custom(lengths_per_row: List[List[int]], hq: int, hkv: int, d: int, dtype: str,
                seed: int) -> Workload:
    """A workload with caller-chosen lengths (tests: ragged tails, tile edges)."""
    T = sum(lengths_per_row[0])
    cfg = Config(0, "custom", len(lengths_per_row), T, hq, hkv, d, dtype, "fixed", (tuple(lengths_per_row[0]),))
    rng = np.random.default_rng(seed)
    pos = position_ids_from_lengths(lengths_per_row)
    N = cfg.n_tokens
    shapes = [(N, hq, d), (N, hkv, d), (N, hkv, d), (N, hq, d)]
    arrs = [rng.standard_normal(s, dtype=np.float32) for s in shapes]
    if dtype == "bf16":
        arrs = [round_to_bf16(a) for a in arrs]
    elif dtype == "f16":
        arrs = [round_to_f16(a) for a in arrs]
    w = Workload(cfg, seed, [list(r) for r in lengths_per_row], pos, *arrs, stats=length_stats(lengths_per_row))
    return w


def padded_layout(lengths_per_row: List[List[int]], group: int = 4, mode: str = "group_max"):
    """Batch-level padding of the same examples (Section 3: a minibatch of `group`
    examples becomes a (group, L_max) tensor, each example right-padded to the
    longest of the group).  Returns a list of (example_length, padded_length)
    in generation order.  mode "global_max" pads every example to the longest
    example of the whole workload instead."""
    flat = [L for row in lengths_per_row for L in row]
    out = []
    if mode == "global_max":
        m = max(flat)
        return [(L, m) for L in flat]
    for s in range(0, len(flat), group):
        g = flat[s:s + group]
        m = max(g)
        out.extend((L, m) for L in g)
    return out
