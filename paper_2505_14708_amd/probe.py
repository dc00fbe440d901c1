"""ctypes binding of the bench's measuring sticks (csrc/probe/da_probe.h, lib/libdaprobe.so).

Not part of the attention path and not in the product library: bench.py uses them to print what this
machine sustains (a matrix-instruction loop, a plain copy, a plain read) beside the published peaks.
"""
from __future__ import annotations

import ctypes
import os

from .binding import _check, _ptr, _stream

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "lib", "libdaprobe.so")
EXPORTS = ["da_probe_mfma_bf16", "da_probe_copy", "da_probe_read"]

_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is not built; run `python -m paper_2505_14708_amd.build` first")
        L = ctypes.CDLL(LIB_PATH)
        V = ctypes.c_void_p
        L.da_probe_mfma_bf16.argtypes = [ctypes.c_int, V, ctypes.POINTER(ctypes.c_double), V]
        L.da_probe_copy.argtypes = [V, V, ctypes.c_size_t, V]
        L.da_probe_read.argtypes = [V, ctypes.c_size_t, V, V]
        for name in EXPORTS:
            getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def da_probe_mfma_bf16(iters: int, sink, stream=None) -> float:
    """Enqueue the matrix-instruction loop; returns the flop one launch performs."""
    flop = ctypes.c_double(0.0)
    _check(lib().da_probe_mfma_bf16(int(iters), _ptr(sink), ctypes.byref(flop), _stream(stream)), "da_probe_mfma_bf16")
    return float(flop.value)


def da_probe_copy(src, dst, nbytes: int, stream=None):
    _check(lib().da_probe_copy(_ptr(src), _ptr(dst), ctypes.c_size_t(int(nbytes)), _stream(stream)), "da_probe_copy")


def da_probe_read(src, nbytes: int, sink, stream=None):
    _check(lib().da_probe_read(_ptr(src), ctypes.c_size_t(int(nbytes)), _ptr(sink), _stream(stream)), "da_probe_read")
