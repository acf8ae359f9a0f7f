"""ctypes binding of libdma_probe.so (include/dma_probe.h): the benchmark's device yardsticks.

Not part of the attention library: a register-resident loop of the MFMA instruction the attention
kernels use, and a streaming copy.  Marshalling only; raises if the library has not been built.
"""
from __future__ import annotations

import ctypes
import os

from .binding import _check, _ptr, _stream

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libdma_probe.so")
_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} not found: build it first (python -c 'import __graft_entry__ as g; g.build()')")
        L = ctypes.CDLL(LIB_PATH)
        vp, sz, i32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
        L.dma_probe_mfma.argtypes = [vp, i32, i32, vp]
        L.dma_probe_mfma.restype = i32
        L.dma_probe_copy.argtypes = [vp, vp, sz, vp]
        L.dma_probe_copy.restype = i32
        _lib = L
    return _lib


def dma_probe_mfma(sink, n_workgroups, iters, stream=None):
    _check(lib().dma_probe_mfma(_ptr(sink), int(n_workgroups), int(iters), _stream(stream)), "dma_probe_mfma")


def dma_probe_copy(src, dst, nbytes, stream=None):
    _check(lib().dma_probe_copy(_ptr(src), _ptr(dst), int(nbytes), _stream(stream)), "dma_probe_copy")
