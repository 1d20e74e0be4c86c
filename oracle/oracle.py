"""ctypes front end of the C oracle (oracle/varlen_oracle.c).  TEST INFRASTRUCTURE ONLY.

Every function takes and returns numpy arrays; floating point is fp64.  The
arithmetic lives in the C file, whose header states the definitions followed
(Section 3 / 3.1 of the paper for the boundaries, Table 1 for the mask, the
textbook softmax-attention definition and its analytic gradients otherwise).
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build()
        _lib = C.CDLL(path)
        _lib.oracle_num_threads.restype = C.c_int
    return _lib


def _p(a, ty):
    return a.ctypes.data_as(C.POINTER(ty))


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def pack(position_ids: np.ndarray):
    """position_ids int [R, T] -> dict(cu_seqlens int32 [n+1], seg_id int32 [N], n, max_seqlen,
    seg_start int32 [N], seg_end int32 [N])."""
    pos = np.ascontiguousarray(position_ids, dtype=np.int64)
    assert pos.ndim == 2
    R, T = pos.shape
    N = R * T
    cu = np.zeros(N + 1, dtype=np.int32)
    seg_id = np.zeros(N, dtype=np.int32)
    n = C.c_int32(0)
    mx = C.c_int32(0)
    rc = lib().oracle_pack(_p(pos, C.c_int64), C.c_int(R), C.c_int(T), _p(cu, C.c_int32),
                           _p(seg_id, C.c_int32), C.byref(n), C.byref(mx))
    if rc != 0:
        raise RuntimeError(f"oracle_pack failed: {rc}")
    cu = cu[: n.value + 1].copy()
    return {
        "cu_seqlens": cu, "seg_id": seg_id, "n": int(n.value), "max_seqlen": int(mx.value),
        "seg_start": cu[seg_id].astype(np.int32), "seg_end": cu[seg_id + 1].astype(np.int32),
    }


def collate(ids_padded, lengths, n_out, labels_padded=None, pad_id=0):
    """Padding-free collator (Section 3.4) on a padded [n, Lp] batch -> dict(input_ids, labels,
    position_ids: int64 [n_out]; offsets int32 [n+1])."""
    ids = np.ascontiguousarray(ids_padded, dtype=np.int64)
    assert ids.ndim == 2
    n, Lp = ids.shape
    lab = None if labels_padded is None else np.ascontiguousarray(labels_padded, dtype=np.int64)
    lengths = np.ascontiguousarray(lengths, dtype=np.int32)
    assert lengths.shape == (n,)
    out = {k: np.full(n_out, -7, dtype=np.int64) for k in ("input_ids", "labels", "position_ids")}
    offsets = np.zeros(n + 1, dtype=np.int32)
    rc = lib().oracle_collate(_p(ids, C.c_int64), None if lab is None else _p(lab, C.c_int64),
                              _p(lengths, C.c_int32), C.c_int(n), C.c_int(Lp), C.c_int64(n_out),
                              C.c_int64(pad_id), _p(out["input_ids"], C.c_int64), _p(out["labels"], C.c_int64),
                              _p(out["position_ids"], C.c_int64), _p(offsets, C.c_int32))
    if rc != 0:
        raise RuntimeError(f"oracle_collate failed: {rc}")
    out["offsets"] = offsets
    return out


def rope(x, position_ids, base=10000.0, inverse=False):
    """Rotary embedding of x [N, H, d] at positions position_ids (any shape with N entries) -> fp64."""
    x = _f64(x)
    N, H, d = x.shape
    pos = np.ascontiguousarray(position_ids, dtype=np.int64).reshape(-1)
    assert pos.shape[0] == N
    y = np.empty_like(x)
    rc = lib().oracle_rope(_p(x, C.c_double), _p(y, C.c_double), _p(pos, C.c_int64), C.c_int64(N), C.c_int(H),
                           C.c_int(d), C.c_double(base), C.c_int(1 if inverse else 0))
    if rc != 0:
        raise RuntimeError(f"oracle_rope failed: {rc}")
    return y


def _dims(q, k):
    N, Hq, d = q.shape
    Nk, Hkv, dk = k.shape
    assert Nk == N and dk == d
    return N, Hq, Hkv, d


def fwd(q, k, v, cu_seqlens, scale=None):
    """-> O [N, Hq, d] fp64, LSE [Hq, N] fp64."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    N, Hq, Hkv, d = _dims(q, k)
    cu = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
    scale = 1.0 / np.sqrt(d) if scale is None else float(scale)
    O = np.empty_like(q)
    LSE = np.empty((Hq, N), dtype=np.float64)
    D = C.POINTER(C.c_double)
    rc = lib().oracle_fwd(_p(q, C.c_double), _p(k, C.c_double), _p(v, C.c_double), _p(cu, C.c_int32),
                          C.c_int(len(cu) - 1), C.c_int(N), C.c_int(Hq), C.c_int(Hkv), C.c_int(d),
                          C.c_double(scale), _p(O, C.c_double), _p(LSE, C.c_double))
    if rc != 0:
        raise RuntimeError(f"oracle_fwd failed: {rc}")
    return O, LSE


def bwd(do, q, k, v, cu_seqlens, scale=None):
    """-> dQ [N, Hq, d], dK [N, Hkv, d], dV [N, Hkv, d], fp64."""
    do, q, k, v = _f64(do), _f64(q), _f64(k), _f64(v)
    N, Hq, Hkv, d = _dims(q, k)
    cu = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
    scale = 1.0 / np.sqrt(d) if scale is None else float(scale)
    dQ = np.empty_like(q)
    dK = np.empty_like(k)
    dV = np.empty_like(v)
    rc = lib().oracle_bwd(_p(do, C.c_double), _p(q, C.c_double), _p(k, C.c_double), _p(v, C.c_double),
                          _p(cu, C.c_int32), C.c_int(len(cu) - 1), C.c_int(N), C.c_int(Hq), C.c_int(Hkv),
                          C.c_int(d), C.c_double(scale), _p(dQ, C.c_double), _p(dK, C.c_double),
                          _p(dV, C.c_double))
    if rc != 0:
        raise RuntimeError(f"oracle_bwd failed: {rc}")
    return dQ, dK, dV


def rows_q(do, q, k, v, cu_seqlens, tok, head, scale=None):
    """Sampled outputs: O[tok, head, :], LSE[head, tok], dQ[tok, head, :] (dQ None if do is None)."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    N, Hq, Hkv, d = _dims(q, k)
    cu = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
    tok = np.ascontiguousarray(tok, dtype=np.int32)
    head = np.ascontiguousarray(head, dtype=np.int32)
    m = len(tok)
    scale = 1.0 / np.sqrt(d) if scale is None else float(scale)
    O = np.empty((m, d), dtype=np.float64)
    LSE = np.empty(m, dtype=np.float64)
    if do is not None:
        do = _f64(do)
        dQ = np.empty((m, d), dtype=np.float64)
        pdo, pdq = _p(do, C.c_double), _p(dQ, C.c_double)
    else:
        dQ, pdo, pdq = None, None, None
    rc = lib().oracle_rows_q(pdo, _p(q, C.c_double), _p(k, C.c_double), _p(v, C.c_double),
                             _p(cu, C.c_int32), C.c_int(len(cu) - 1), C.c_int(N), C.c_int(Hq), C.c_int(Hkv),
                             C.c_int(d), C.c_double(scale), _p(tok, C.c_int32), _p(head, C.c_int32),
                             C.c_int(m), _p(O, C.c_double), _p(LSE, C.c_double), pdq)
    if rc != 0:
        raise RuntimeError(f"oracle_rows_q failed: {rc}")
    return O, LSE, dQ


def rows_kv(do, q, k, v, cu_seqlens, tok, kvhead, scale=None):
    """Sampled outputs: dK[tok, kvhead, :], dV[tok, kvhead, :]."""
    do, q, k, v = _f64(do), _f64(q), _f64(k), _f64(v)
    N, Hq, Hkv, d = _dims(q, k)
    cu = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
    tok = np.ascontiguousarray(tok, dtype=np.int32)
    kvhead = np.ascontiguousarray(kvhead, dtype=np.int32)
    m = len(tok)
    scale = 1.0 / np.sqrt(d) if scale is None else float(scale)
    dK = np.empty((m, d), dtype=np.float64)
    dV = np.empty((m, d), dtype=np.float64)
    rc = lib().oracle_rows_kv(_p(do, C.c_double), _p(q, C.c_double), _p(k, C.c_double), _p(v, C.c_double),
                              _p(cu, C.c_int32), C.c_int(len(cu) - 1), C.c_int(N), C.c_int(Hq), C.c_int(Hkv),
                              C.c_int(d), C.c_double(scale), _p(tok, C.c_int32), _p(kvhead, C.c_int32),
                              C.c_int(m), _p(dK, C.c_double), _p(dV, C.c_double))
    if rc != 0:
        raise RuntimeError(f"oracle_rows_kv failed: {rc}")
    return dK, dV
