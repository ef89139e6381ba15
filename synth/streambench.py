"""ctypes access to the harness's bandwidth probes (synth/csrc/streambench.hip): a K-stream read-only kernel and a copy
kernel, timed with HIP events on the device.  Harness only: none of the parameter server's work."""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(_HERE, "csrc", "streambench.hip")
LIB = os.path.join(_HERE, "libsynth_streambench.so")
READ_STREAM_COUNTS = (1, 2, 3, 4, 8, 16, 20, 32)
_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB):
            raise RuntimeError(f"{LIB} missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
        _lib = C.CDLL(LIB)
        _lib.synth_stream_read.argtypes = [C.POINTER(C.c_void_p), C.c_uint32, C.c_uint64, C.c_void_p, C.c_uint32, C.c_void_p,
                                           C.POINTER(C.c_float)]
        _lib.synth_stream_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.c_uint32, C.c_void_p, C.POINTER(C.c_float)]
        _lib.synth_stream_read.restype = _lib.synth_stream_copy.restype = C.c_int
    return _lib


def read_gbps(stream_ptrs, n, sink_ptr, reps=20, stream=0):
    """GB/s of a read-only pass over len(stream_ptrs) vectors of n floats (device addresses)."""
    arr = (C.c_void_p * len(stream_ptrs))(*stream_ptrs)
    ms = C.c_float()
    rc = lib().synth_stream_read(arr, len(stream_ptrs), n, sink_ptr, reps, stream or None, C.byref(ms))
    if rc != 0:
        raise RuntimeError(f"synth_stream_read failed with hipError {rc}")
    return 4.0 * n * len(stream_ptrs) / (ms.value * 1e-3) / 1e9


def copy_gbps(src_ptr, dst_ptr, n, reps=20, stream=0):
    """GB/s (bytes read + bytes written) of a plain copy of n floats."""
    ms = C.c_float()
    rc = lib().synth_stream_copy(src_ptr, dst_ptr, n, reps, stream or None, C.byref(ms))
    if rc != 0:
        raise RuntimeError(f"synth_stream_copy failed with hipError {rc}")
    return 8.0 * n / (ms.value * 1e-3) / 1e9
