"""Binding of libvq_bench.so, the benchmark's HBM read probe (include/vq_bench.h).  Not part of
the product: nothing in the package's hot path imports this module."""
from __future__ import annotations

import ctypes
import os

from . import VQError, _ptr, _stream

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libvq_bench.so")
_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(f"{_LIB_PATH} is not built; run `python -m paper_2402_15319_amd.build`")
        L = ctypes.CDLL(_LIB_PATH)
        L.vq_bench_stream_read.restype = ctypes.c_int
        L.vq_bench_stream_read.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        _lib = L
    return _lib


def vq_bench_stream_read(buf, nbytes: int, stream=None) -> None:
    st = lib().vq_bench_stream_read(_ptr(buf), nbytes, _stream(stream))
    if st != 0:
        raise VQError(st, "vq_bench_stream_read")
