"""Loader of libespn_benchprobe.so: the benchmark's measuring sticks (a plain streaming read, a plain copy of
known size).  Not part of the re-ranking library or of its header; bench.py and one GPU test use it."""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libespn_benchprobe.so")
_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("%s is missing: build it with `python -m paper_2312_05417_amd.build`" % LIB_PATH)
        handle = ctypes.CDLL(LIB_PATH)
        handle.espn_bench_stream_read.restype = ctypes.c_int
        handle.espn_bench_stream_read.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p]
        handle.espn_bench_copy.restype = ctypes.c_int
        handle.espn_bench_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        _lib = handle
    return _lib


def stream_read(src_ptr: int, nbytes: int, sink_ptr: int, stream_ptr: int) -> None:
    rc = lib().espn_bench_stream_read(src_ptr, nbytes, sink_ptr, stream_ptr)
    if rc != 0:
        raise ValueError("espn_bench_stream_read: %s" % ("bad argument" if rc == 1 else "launch failed"))


def copy(src_ptr: int, dst_ptr: int, nbytes: int, stream_ptr: int) -> None:
    rc = lib().espn_bench_copy(src_ptr, dst_ptr, nbytes, stream_ptr)
    if rc != 0:
        raise ValueError("espn_bench_copy: %s" % ("bad argument" if rc == 1 else "launch failed"))
