"""Counter-based synthetic vectors: initial weights and learner gradients.

Seeded INPUT generator shared by the CPU oracle's tests and the GPU runs.  It
holds none of the parameter server's arithmetic: it only manufactures the
numbers a learner's calcGradient would have produced (the paper's data sets and
networks are not available; only its vector sizes and learner counts are used).

Every value is a pure function of (seed, tag, learner, step, index):

    key  = mix(mix(mix(seed ^ tag*K_TAG) + learner) + step)          64-bit
    u    = key + index * GOLDEN                                       64-bit wrap
    a, b = mix(u), mix(u ^ K_SECOND)
    S    = sum of the eight 16-bit lanes of a and b                   0 .. 8*65535
    x    = float32(S - 4*65535) * scale                               one binary32 multiply

S is an Irwin-Hall sum (mean 4*65535, variance 8*(65536^2-1)/12), so x is close
to N(0, std^2) with std = scale * IH_STD, cut off at +-4.9 std.  No libm call is
involved, so the host (numpy, below) and the device kernel (csrc/gradgen.hip)
produce identical bits.  With tail_per = T > 0 an entry is multiplied by
tail_factor with probability 1/T (decided by a third hash): the heavy tail of
the 72M-parameter workload.

`mix` is the splitmix64 output function (Steele, Lea, Flood 2014).
"""
from __future__ import annotations

import ctypes as C
import math
import os

import numpy as np

MASK = (1 << 64) - 1
GOLDEN = 0x9E3779B97F4A7C15
K_TAG = 0xC2B2AE3D27D4EB4F
K_SECOND = 0xD1B54A32D192ED03
K_TAIL = 0x8CB92BA72F3D8DD7
IH_MEAN = 4 * 65535
IH_STD = math.sqrt(8 * (65536.0 ** 2 - 1.0) / 12.0)

TAG_INIT, TAG_GRAD, TAG_TIME, TAG_STRAGGLER = 1, 2, 3, 4


def mix_int(x: int) -> int:
    x &= MASK
    x ^= x >> 30
    x = (x * 0xBF58476D1CE4E5B9) & MASK
    x ^= x >> 27
    x = (x * 0x94D049BB133111EB) & MASK
    x ^= x >> 31
    return x


def stream_key(seed: int, tag: int, learner: int = 0, step: int = 0) -> int:
    k = mix_int((seed ^ (tag * K_TAG)) & MASK)
    k = mix_int((k + learner) & MASK)
    k = mix_int((k + step) & MASK)
    return k


def _mix_np(x):
    x = x ^ (x >> np.uint64(30))
    x = x * np.uint64(0xBF58476D1CE4E5B9)
    x = x ^ (x >> np.uint64(27))
    x = x * np.uint64(0x94D049BB133111EB)
    x = x ^ (x >> np.uint64(31))
    return x


def _lanes(h):
    m = np.uint64(0xFFFF)
    return (h & m) + ((h >> np.uint64(16)) & m) + ((h >> np.uint64(32)) & m) + (h >> np.uint64(48))


def scales(std: float, tail_factor: float = 1.0):
    """(scale, scale_tail) as binary32: computed once on the host, handed to both sides."""
    return np.float32(std / IH_STD), np.float32(std * tail_factor / IH_STD)


def values_at(key: int, index, std: float, tail_per: int = 0, tail_factor: float = 100.0):
    """float32 values of the stream `key` at the given indices (any integer array)."""
    idx = np.asarray(index, dtype=np.uint64)
    with np.errstate(over="ignore"):
        u = np.uint64(key) + idx * np.uint64(GOLDEN)
        a = _mix_np(u)
        b = _mix_np(u ^ np.uint64(K_SECOND))
        s = (_lanes(a) + _lanes(b)).astype(np.int64) - IH_MEAN
        scale, scale_tail = scales(std, tail_factor)
        x = s.astype(np.float32)
        if tail_per:
            t = _mix_np(u + np.uint64(K_TAIL))
            hit = (((t >> np.uint64(32)) * np.uint64(tail_per)) >> np.uint64(32)) == 0
            return np.where(hit, x * scale_tail, x * scale).astype(np.float32)
        return (x * scale).astype(np.float32)


def vector(key: int, n: int, std: float, tail_per: int = 0, tail_factor: float = 100.0, chunk: int = 1 << 22):
    """The whole stream 0..n-1 on the host (chunked to bound temporaries)."""
    out = np.empty(n, dtype=np.float32)
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        out[lo:hi] = values_at(key, np.arange(lo, hi, dtype=np.uint64), std, tail_per, tail_factor)
    return out


def uniform01(seed: int, tag: int, learner: int, step: int) -> float:
    """One double in (0, 1] for the arrival-time draws (host only)."""
    h = stream_key(seed, tag, learner, step)
    return ((h >> 11) + 1) / float(1 << 53)


# ---------------------------------------------------------------------------
# device twin
# ---------------------------------------------------------------------------
_HERE = os.path.dirname(os.path.abspath(__file__))
DEVICE_SRC = os.path.join(_HERE, "csrc", "gradgen.hip")
DEVICE_LIB = os.path.join(_HERE, "libsynth_gradgen.so")
_dev = None


def device_lib():
    """ctypes handle of the device generator (must have been built beforehand)."""
    global _dev
    if _dev is None:
        if not os.path.exists(DEVICE_LIB):
            raise RuntimeError(f"{DEVICE_LIB} missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
        _dev = C.CDLL(DEVICE_LIB)
        _dev.synth_fill.argtypes = [C.c_void_p, C.c_uint64, C.c_uint64, C.c_float, C.c_float, C.c_uint32, C.c_void_p]
        _dev.synth_fill.restype = C.c_int
    return _dev


def fill_device(dst_ptr: int, n: int, key: int, std: float, tail_per: int = 0, tail_factor: float = 100.0,
                stream: int = 0):
    """Enqueue the generator kernel on `stream`: dst[0..n) = stream `key` (device pointer, 16-byte aligned)."""
    scale, scale_tail = scales(std, tail_factor)
    rc = device_lib().synth_fill(dst_ptr, n, key, float(scale), float(scale_tail), tail_per, stream)
    if rc != 0:
        raise RuntimeError(f"synth_fill failed with hipError {rc}")
