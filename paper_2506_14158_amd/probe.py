"""ctypes binding of libs4c_probe.so: the benchmark's measurement probes (plain streaming read, plain
matrix-core loop).  Not part of the verification library; only bench.py loads it."""
from __future__ import annotations

import ctypes as C
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libs4c_probe.so")
_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError("%s not found: build it first (python -c 'import __graft_entry__ as g; g.build()')" % LIB_PATH)
        L = C.CDLL(LIB_PATH)
        L.s4c_probe_stream_read.restype = C.c_int
        L.s4c_probe_stream_read.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
        L.s4c_probe_mfma_sink_bytes.restype = C.c_size_t
        L.s4c_probe_mfma_sink_bytes.argtypes = []
        L.s4c_probe_mfma_bf16.restype = C.c_int
        L.s4c_probe_mfma_bf16.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.POINTER(C.c_double), C.c_void_p]
        _lib = L
    return _lib


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def mfma_sink(device="cuda") -> torch.Tensor:
    return torch.zeros(lib().s4c_probe_mfma_sink_bytes() // 4, dtype=torch.float32, device=device)


def stream_read(buffer: torch.Tensor, sink: torch.Tensor) -> None:
    """Enqueue one streaming read of `buffer` (time it with events)."""
    rc = lib().s4c_probe_stream_read(buffer.data_ptr(), buffer.numel() * buffer.element_size(), sink.data_ptr(), _stream())
    if rc != 0:
        raise RuntimeError("s4c_probe_stream_read failed (%d)" % rc)


def mfma_bf16(random_operands: bool, iters: int, sink: torch.Tensor, shape: int = 0) -> float:
    """Enqueue the matrix-core probe (shape 0: 32x32x16, 1: 16x16x32); returns the FLOP count of the launch."""
    if sink.numel() * sink.element_size() < lib().s4c_probe_mfma_sink_bytes():
        raise ValueError("sink too small")
    flops = C.c_double(0.0)
    rc = lib().s4c_probe_mfma_bf16(int(bool(random_operands)), int(shape), int(iters), sink.data_ptr(), C.byref(flops), _stream())
    if rc != 0:
        raise RuntimeError("s4c_probe_mfma_bf16 failed (%d)" % rc)
    return float(flops.value)
