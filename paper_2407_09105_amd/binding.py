"""Thin ctypes binding of libvarlen_attn.so (include/varlen_attn.h).

Argument marshalling only: every step of the path (boundary scan, tile schedule,
forward, backward) runs in the library's HIP kernels.  PyTorch supplies device
memory and the stream.  There is no fallback: if the library is missing, or a
call returns a non-zero status, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libvarlen_attn.so")

VA_OK = 0
VA_F32, VA_BF16, VA_F16 = 0, 1, 2
VA_I32, VA_I64 = 0, 1
VA_TILE = 256
STAGE_D, STAGE_DKDV, STAGE_DQ = 1, 2, 4
HINT_LONG_EXAMPLES, HINT_SHORT_EXAMPLES = 8, 16

EXPORTS = (
    "va_plan_bytes", "va_segments_bind", "va_pack_to_cu_seqlens", "va_attn_workspace_bytes",
    "va_varlen_attn_fwd", "va_varlen_attn_bwd", "va_varlen_attn_bwd_stages", "va_varlen_attn_bwd_noalloc",
    "va_collate_padding_free",
    "va_rope_apply", "va_status_string", "va_version",
)


class VaSegments(C.Structure):
    _fields_ = [(name, C.c_void_p) for name in (
        "cu_seqlens", "seg_id", "seg_start", "seg_end", "meta", "q_tile_order", "kv_tile_order", "scratch")]


_lib = None


def lib() -> C.CDLL:
    """Load the built library (build it first with `python -m paper_2407_09105_amd.build`)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built; run __graft_entry__.build() "
                          "(python paper_2407_09105_amd/build.py)")
    L = C.CDLL(LIB_PATH)
    L.va_plan_bytes.restype = C.c_size_t
    L.va_plan_bytes.argtypes = [C.c_int32, C.c_int32]
    L.va_segments_bind.restype = C.c_int
    L.va_segments_bind.argtypes = [C.c_void_p, C.c_size_t, C.c_int32, C.c_int32, C.POINTER(VaSegments)]
    L.va_pack_to_cu_seqlens.restype = C.c_int
    L.va_pack_to_cu_seqlens.argtypes = [C.c_void_p, C.c_int, C.c_int32, C.c_int32, C.POINTER(VaSegments),
                                        C.c_void_p]
    L.va_attn_workspace_bytes.restype = C.c_size_t
    L.va_attn_workspace_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int]
    L.va_varlen_attn_fwd.restype = C.c_int
    L.va_varlen_attn_fwd.argtypes = [C.c_void_p] * 5 + [C.POINTER(VaSegments)] + [C.c_int32] * 5 + [
        C.c_int, C.c_float, C.c_void_p, C.c_size_t, C.c_void_p]
    L.va_varlen_attn_bwd.restype = C.c_int
    L.va_varlen_attn_bwd.argtypes = [C.c_void_p] * 9 + [C.c_int, C.POINTER(VaSegments)] + [C.c_int32] * 5 + [
        C.c_int, C.c_float, C.c_void_p, C.c_size_t, C.c_void_p]
    L.va_varlen_attn_bwd_stages.restype = C.c_int
    L.va_varlen_attn_bwd_stages.argtypes = L.va_varlen_attn_bwd.argtypes + [C.c_uint32]
    L.va_varlen_attn_bwd_noalloc.restype = C.c_int
    L.va_varlen_attn_bwd_noalloc.argtypes = [C.c_void_p] * 9 + [C.c_int, C.POINTER(VaSegments)] + [C.c_int32] * 5 + [
        C.c_int, C.c_float, C.c_void_p]
    L.va_collate_padding_free.restype = C.c_int
    L.va_collate_padding_free.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_int32, C.c_int32,
                                          C.c_int32, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p,
                                          C.c_void_p, C.c_void_p]
    L.va_rope_apply.restype = C.c_int
    L.va_rope_apply.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_int32, C.c_int32,
                                C.c_int32, C.c_float, C.c_int, C.c_void_p]
    L.va_status_string.restype = C.c_char_p
    L.va_status_string.argtypes = [C.c_int]
    L.va_version.restype = C.c_char_p
    _lib = L
    return L


class VarlenAttnError(RuntimeError):
    def __init__(self, what: str, status: int):
        self.status = status
        super().__init__(f"{what}: {lib().va_status_string(status).decode()} (status {status})")


def _check(what: str, status: int):
    if status != VA_OK:
        raise VarlenAttnError(what, status)


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return VA_F32
    if t.dtype == torch.bfloat16:
        return VA_BF16
    if t.dtype == torch.float16:
        return VA_F16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _need_cuda(*ts):
    for t in ts:
        if not t.is_cuda:
            raise ValueError("tensors must live on the GPU")
        if not t.is_contiguous():
            raise ValueError("tensors must be contiguous")


class Segments:
    """Device-side example boundaries and tile schedule of one packed stream."""

    def __init__(self, rows: int, tokens_per_row: int, device):
        self.rows, self.tokens_per_row = int(rows), int(tokens_per_row)
        self.n_tokens = self.rows * self.tokens_per_row
        nbytes = lib().va_plan_bytes(self.rows, self.tokens_per_row)
        if nbytes == 0:
            raise VarlenAttnError("va_plan_bytes", 2)
        self.plan = torch.empty(nbytes // 4, dtype=torch.int32, device=device)
        self.c = VaSegments()
        _check("va_segments_bind", lib().va_segments_bind(self.plan.data_ptr(), nbytes, self.rows,
                                                          self.tokens_per_row, C.byref(self.c)))

    def _view(self, ptr: int, count: int) -> torch.Tensor:
        off = (ptr - self.plan.data_ptr()) // 4
        return self.plan[off: off + count]

    # Views into the plan buffer (device tensors; reading them on the host synchronises).
    @property
    def n_tiles(self) -> int:
        return self.rows * ((self.tokens_per_row + VA_TILE - 1) // VA_TILE)

    @property
    def meta(self): return self._view(self.c.meta, 8)
    @property
    def seg_id(self): return self._view(self.c.seg_id, self.n_tokens)
    @property
    def seg_start(self): return self._view(self.c.seg_start, self.n_tokens)
    @property
    def seg_end(self): return self._view(self.c.seg_end, self.n_tokens)
    @property
    def cu_seqlens_capacity(self): return self._view(self.c.cu_seqlens, self.n_tokens + 1)
    @property
    def q_tile_order(self): return self._view(self.c.q_tile_order, self.n_tiles)
    @property
    def kv_tile_order(self): return self._view(self.c.kv_tile_order, self.n_tiles)

    def host(self) -> dict:
        """Copy the results to the host (synchronises): cu_seqlens[:n+1], n, max_seqlen, seg arrays."""
        meta = self.meta.cpu()
        n = int(meta[0])
        return {
            "n": n, "max_seqlen": int(meta[1]),
            "cu_seqlens": self.cu_seqlens_capacity[: n + 1].cpu().numpy(),
            "seg_id": self.seg_id.cpu().numpy(), "seg_start": self.seg_start.cpu().numpy(),
            "seg_end": self.seg_end.cpu().numpy(),
            # order entries: tile index in bits 0..23, the tile's head rotation above
            "q_tile_order": self.q_tile_order.cpu().numpy() & 0xFFFFFF, "kv_tile_order": self.kv_tile_order.cpu().numpy() & 0xFFFFFF,
            "q_tile_rotation": self.q_tile_order.cpu().numpy() >> 24, "kv_tile_rotation": self.kv_tile_order.cpu().numpy() >> 24,
        }


def pack_to_cu_seqlens(position_ids: torch.Tensor, seg: Optional[Segments] = None) -> Segments:
    """position_ids [R, T] (int32 or int64, GPU) -> Segments.  Enqueues kernels only."""
    _need_cuda(position_ids)
    if position_ids.dim() != 2:
        raise ValueError("position_ids must be [rows, tokens_per_row]")
    if position_ids.dtype == torch.int64:
        it = VA_I64
    elif position_ids.dtype == torch.int32:
        it = VA_I32
    else:
        raise TypeError("position_ids must be int32 or int64")
    R, T = position_ids.shape
    if seg is None:
        seg = Segments(R, T, position_ids.device)
    elif (seg.rows, seg.tokens_per_row) != (R, T):
        raise ValueError("Segments object was made for another shape")
    _check("va_pack_to_cu_seqlens",
           lib().va_pack_to_cu_seqlens(position_ids.data_ptr(), it, R, T, C.byref(seg.c), _stream()))
    return seg


def collate_padding_free(ids_padded: torch.Tensor, lengths: torch.Tensor, n_out: int,
                         labels_padded: Optional[torch.Tensor] = None, pad_id: int = 0, out=None):
    """Padded batch [n, Lp] + lengths [n] (int32) -> dict(input_ids, labels, position_ids: [1, n_out]
    of the ids' dtype; example_offsets int32 [n + 1]).  Enqueues kernels only."""
    _need_cuda(ids_padded, lengths)
    if ids_padded.dim() != 2 or lengths.dim() != 1 or lengths.shape[0] != ids_padded.shape[0]:
        raise ValueError("expected ids_padded [n, Lp] and lengths [n]")
    if ids_padded.dtype not in (torch.int32, torch.int64) or lengths.dtype != torch.int32:
        raise TypeError("ids must be int32 or int64, lengths int32")
    if labels_padded is not None:
        _need_cuda(labels_padded)
        if labels_padded.shape != ids_padded.shape or labels_padded.dtype != ids_padded.dtype:
            raise ValueError("labels_padded must match ids_padded")
    n, Lp = ids_padded.shape
    it = VA_I64 if ids_padded.dtype == torch.int64 else VA_I32
    dev = ids_padded.device
    if out is None:
        out = {k: torch.empty((1, n_out), dtype=ids_padded.dtype, device=dev)
               for k in ("input_ids", "labels", "position_ids")}
        out["example_offsets"] = torch.empty(n + 1, dtype=torch.int32, device=dev)
    else:
        for key in ("input_ids", "labels", "position_ids"):
            if out[key].numel() != n_out:
                raise ValueError(f"out[{key!r}] must hold n_out = {n_out} elements")
            _out_like(f"out[{key!r}]", out[key], out[key].shape, ids_padded.dtype, dev)
        _out_like("out['example_offsets']", out["example_offsets"], (n + 1,), torch.int32, dev)
    _check("va_collate_padding_free", lib().va_collate_padding_free(
        ids_padded.data_ptr() if n else None, None if labels_padded is None else labels_padded.data_ptr(), it,
        lengths.data_ptr() if n else None, n, Lp, n_out, int(pad_id), out["input_ids"].data_ptr(),
        out["labels"].data_ptr(), out["position_ids"].data_ptr(), out["example_offsets"].data_ptr(), _stream()))
    return out


def rope_apply(x: torch.Tensor, position_ids: torch.Tensor, theta_base: float = 10000.0, inverse: bool = False,
               out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Rotary embedding of x [N, H, d] (float32, bfloat16 or float16) at position_ids (N entries, int32/int64).
    out may be x (in place).  Enqueues one kernel."""
    _need_cuda(x, position_ids)
    if x.dim() != 3 or position_ids.numel() != x.shape[0]:
        raise ValueError("expected x [N, H, d] and N position ids")
    if position_ids.dtype not in (torch.int32, torch.int64):
        raise TypeError("position_ids must be int32 or int64")
    y = torch.empty_like(x) if out is None else out
    if y.shape != x.shape or y.dtype != x.dtype:
        raise ValueError("out must match x")
    _need_cuda(y)
    N, H, d = x.shape
    _check("va_rope_apply", lib().va_rope_apply(
        x.data_ptr(), y.data_ptr(), _dt(x), position_ids.data_ptr(),
        VA_I64 if position_ids.dtype == torch.int64 else VA_I32, N, H, d, float(theta_base), int(inverse), _stream()))
    return y


def _out_like(name: str, t: torch.Tensor, shape, dtype, device):
    """A caller-supplied output buffer must be exactly what the library will write: it only gets the pointer."""
    _need_cuda(t)
    if tuple(t.shape) != tuple(shape) or t.dtype != dtype or t.device != device:
        raise ValueError(f"{name} must be a contiguous {dtype} tensor of shape {tuple(shape)} on {device}, "
                         f"got {t.dtype} {tuple(t.shape)} on {t.device}")
    return t


def _shapes(q, k, v, seg):
    if q.dim() != 3 or k.dim() != 3 or v.shape != k.shape:
        raise ValueError("expected Q [N, Hq, d], K/V [N, Hkv, d]")
    N, hq, d = q.shape
    if k.shape[0] != N or k.shape[2] != d or N != seg.n_tokens:
        raise ValueError("token counts / head_dim of Q, K, V and the Segments disagree")
    return N, hq, k.shape[1], d


def varlen_attn_fwd(q, k, v, seg: Segments, softmax_scale: float = 0.0, out=None, lse=None
                    ) -> Tuple[torch.Tensor, torch.Tensor]:
    """-> O [N, Hq, d] (dtype of q), LSE [Hq, N] float32."""
    _need_cuda(q, k, v)
    N, hq, hkv, d = _shapes(q, k, v, seg)
    if not (q.dtype == k.dtype == v.dtype):
        raise TypeError("Q, K, V must share a dtype")
    o = torch.empty_like(q) if out is None else _out_like("out", out, q.shape, q.dtype, q.device)
    lse = (torch.empty((hq, N), dtype=torch.float32, device=q.device) if lse is None
           else _out_like("lse", lse, (hq, N), torch.float32, q.device))
    _check("va_varlen_attn_fwd", lib().va_varlen_attn_fwd(
        q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse.data_ptr(), C.byref(seg.c),
        seg.rows, seg.tokens_per_row, hq, hkv, d, _dt(q), float(softmax_scale), None, 0, _stream()))
    return o, lse


def bwd_workspace(q, k) -> torch.Tensor:
    N, hq, d = q.shape
    nbytes = lib().va_attn_workspace_bytes(N, hq, k.shape[1], d, 1)
    return torch.empty(max(nbytes, 4) // 4, dtype=torch.float32, device=q.device)


def varlen_attn_bwd(do, q, k, v, o, lse, seg: Segments, softmax_scale: float = 0.0,
                    grad_dtype: Optional[torch.dtype] = None, dq=None, dk=None, dv=None, workspace=None,
                    stages: Optional[int] = None):
    """-> dQ [N, Hq, d], dK, dV [N, Hkv, d] in grad_dtype (default: dtype of q).
    `stages` (an OR of STAGE_D, STAGE_DKDV, STAGE_DQ, optionally with HINT_LONG_EXAMPLES or
    HINT_SHORT_EXAMPLES) runs only those kernels of the backward."""
    _need_cuda(do, q, k, v, o, lse)
    N, hq, hkv, d = _shapes(q, k, v, seg)
    if not (q.dtype == k.dtype == v.dtype == o.dtype == do.dtype):
        raise TypeError("dO, Q, K, V, O must share a dtype")
    if lse.dtype != torch.float32 or tuple(lse.shape) != (hq, N):
        raise ValueError("LSE must be float32 [Hq, N]")
    given = [t for t in (dq, dk, dv) if t is not None]
    gdt = grad_dtype if grad_dtype is not None else (given[0].dtype if given else q.dtype)
    dq = torch.empty(q.shape, dtype=gdt, device=q.device) if dq is None else _out_like("dq", dq, q.shape, gdt, q.device)
    dk = torch.empty(k.shape, dtype=gdt, device=q.device) if dk is None else _out_like("dk", dk, k.shape, gdt, q.device)
    dv = torch.empty(v.shape, dtype=gdt, device=q.device) if dv is None else _out_like("dv", dv, v.shape, gdt, q.device)
    if workspace is None:
        ws = bwd_workspace(q, k)
    else:
        ws = workspace
        _need_cuda(ws)
        need = lib().va_attn_workspace_bytes(N, hq, hkv, d, 1)
        if ws.dtype != torch.float32 or ws.numel() * 4 < need or ws.device != q.device:
            raise ValueError(f"workspace must be a contiguous float32 tensor of at least {need} bytes on {q.device}")
    args = [do.data_ptr(), q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse.data_ptr(),
            dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), _dt(dq), C.byref(seg.c), seg.rows, seg.tokens_per_row,
            hq, hkv, d, _dt(q), float(softmax_scale), ws.data_ptr(), ws.numel() * 4, _stream()]
    if stages is None:
        _check("va_varlen_attn_bwd", lib().va_varlen_attn_bwd(*args))
    else:
        _check("va_varlen_attn_bwd_stages", lib().va_varlen_attn_bwd_stages(*args, int(stages)))
    return dq, dk, dv


NOALLOC_SCRATCH_BYTES = 32 << 20


def varlen_attn_bwd_noalloc(do, q, k, v, o, lse, seg: Segments, dq, dk, dv, softmax_scale: float = 0.0):
    """The backward through the entry point that allocates nothing: the caller passes every output,
    D lives in the library's own device array (N * Hq * 4 <= NOALLOC_SCRATCH_BYTES).  No tensor is
    created here either."""
    _need_cuda(do, q, k, v, o, lse, dq, dk, dv)
    N, hq, hkv, d = _shapes(q, k, v, seg)
    if not (q.dtype == k.dtype == v.dtype == o.dtype == do.dtype):
        raise TypeError("dO, Q, K, V, O must share a dtype")
    if lse.dtype != torch.float32 or tuple(lse.shape) != (hq, N):
        raise ValueError("LSE must be float32 [Hq, N]")
    _out_like("dq", dq, q.shape, dq.dtype, q.device)
    _out_like("dk", dk, k.shape, dq.dtype, q.device)
    _out_like("dv", dv, v.shape, dq.dtype, q.device)
    _check("va_varlen_attn_bwd_noalloc", lib().va_varlen_attn_bwd_noalloc(
        do.data_ptr(), q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse.data_ptr(),
        dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), _dt(dq), C.byref(seg.c), seg.rows, seg.tokens_per_row,
        hq, hkv, d, _dt(q), float(softmax_scale), _stream()))
    return dq, dk, dv
