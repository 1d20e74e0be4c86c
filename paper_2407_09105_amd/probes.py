"""ctypes binding of libva_probes.so (probes/va_probes.h): the benchmark's measurement aids.
Not part of the attention library; bench.py uses them for its `measured_peaks`."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libva_probes.so")
EXPORTS = ("vap_probe_mfma", "vap_probe_mix")
_lib = None


class ProbeError(RuntimeError):
    pass


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built; run __graft_entry__.build()")
        L = C.CDLL(LIB_PATH)
        L.vap_probe_mfma.restype = C.c_int
        L.vap_probe_mfma.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_double), C.c_void_p]
        L.vap_probe_mix.restype = C.c_int
        L.vap_probe_mix.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32,
                                    C.POINTER(C.c_double), C.c_void_p]
        _lib = L
    return _lib


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def probe_mfma(sink: torch.Tensor, iters: int) -> float:
    """Enqueue the matrix-instruction-only kernel; returns the FLOPs it performs (time it with events)."""
    if not sink.is_cuda or sink.dtype != torch.float32 or sink.numel() < 64:
        raise ValueError("sink must hold at least 64 float32 on the device")
    fl = C.c_double(0.0)
    st = lib().vap_probe_mfma(sink.data_ptr(), int(iters), C.byref(fl), _stream())
    if st != 0:
        raise ProbeError(f"vap_probe_mfma: status {st}")
    return fl.value


def probe_mix(operands: torch.Tensor, lds_reads: int, valu_groups: int, sink: torch.Tensor,
              clocks: Optional[torch.Tensor], iters: int) -> float:
    """Enqueue the matrix + LDS + vector-ALU mix kernel; returns its matrix FLOPs (time it with events).
    operands: >= 64 KB of 16-bit values on the device; clocks: 2 x int64 on the device or None."""
    if not operands.is_cuda or operands.numel() * operands.element_size() < 65536:
        raise ValueError("operands must hold at least 64 KB on the device")
    if not sink.is_cuda or sink.dtype != torch.float32 or sink.numel() < 64:
        raise ValueError("sink must hold at least 64 float32 on the device")
    if clocks is not None and (clocks.dtype != torch.int64 or clocks.numel() < 2 or not clocks.is_cuda):
        raise ValueError("clocks must hold 2 int64 on the device")
    fl = C.c_double(0.0)
    st = lib().vap_probe_mix(operands.data_ptr(), int(lds_reads), int(valu_groups), sink.data_ptr(),
                             clocks.data_ptr() if clocks is not None else None, int(iters), C.byref(fl), _stream())
    if st != 0:
        raise ProbeError(f"vap_probe_mix: status {st}")
    return fl.value
