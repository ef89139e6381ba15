"""CPU oracle of the Rudra parameter-server update path (TEST INFRASTRUCTURE).

Thin ctypes access to ``rudra_oracle.c`` (all arithmetic lives there).  Only
tests/, ``__graft_entry__.smoke()`` and ``bench.py``'s cpu_baseline leg import
this package; it imports nothing from the HIP package and vice versa.

``OraclePS(precision=32)`` is the parity reference (binary32 state, the storage
type the paper names in Sec. 4.2); ``precision=64`` is the same sequence of
steps in binary64.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rudra_oracle.c")
_LIB = os.path.join(_HERE, "librudra_oracle.so")

HARDSYNC, SOFTSYNC = 0, 1
LR_CONST, LR_STATIC_N, LR_AVG_STALENESS, LR_PER_GRADIENT = 0, 1, 2, 3
OPT_SGD, OPT_ADAGRAD = 0, 1
OK, EINVAL, EFUTURE_TS, EHARDSYNC_STALE, EHARDSYNC_DUP, ENOMEM = 0, -1, -2, -3, -4, -5

# every floating-point operation rounded on its own, no value-changing rewrites
CFLAGS = ["-O2", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-std=c11", "-Wall", "-Wextra"]


def build(force: bool = False, src: str = _SRC, out: str = _LIB) -> str:
    """Compile the oracle twice (binary32 and binary64 state) into one shared object."""
    if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(src):
        return out
    objs = []
    for real, prefix in (("float", "oracle32_"), ("double", "oracle64_")):
        obj = out + f".{prefix}.o"
        cmd = ["gcc", *CFLAGS, f"-DORACLE_REAL={real}", f"-DORACLE_PREFIX={prefix}", "-c", src, "-o", obj]
        subprocess.run(cmd, check=True)
        objs.append(obj)
    subprocess.run(["gcc", "-shared", "-o", out, *objs, "-lm"], check=True)
    for o in objs:
        os.remove(o)
    return out


class _Config(C.Structure):
    _fields_ = [("n_params", C.c_uint64), ("n_learners", C.c_uint32), ("n_split", C.c_uint32),
                ("c_override", C.c_uint32), ("protocol", C.c_int32), ("lr_mode", C.c_int32),
                ("alpha0", C.c_float), ("lr_scale", C.c_float), ("momentum", C.c_float),
                ("weight_decay", C.c_float), ("optimizer", C.c_int32), ("adagrad_eps", C.c_float),
                ("max_aggregate", C.c_uint32)]


class PushResult(C.Structure):
    _fields_ = [("staleness", C.c_uint64), ("ts_after", C.c_uint64), ("pending", C.c_uint32),
                ("applied", C.c_int32), ("lr_used", C.c_float)]


_lib = None


def _load():
    global _lib
    if _lib is None:
        # RUDRA_ORACLE_LIB: a prebuilt variant of this same source (the mutation test plants mistakes in copies
        # of rudra_oracle.c and checks that the pins catch them)
        _lib = C.CDLL(os.environ.get("RUDRA_ORACLE_LIB") or build())
        for p in ("oracle32_", "oracle64_"):
            f = lambda n: getattr(_lib, p + n)
            f("create").argtypes = [C.POINTER(_Config), C.c_void_p, C.POINTER(C.c_void_p)]
            f("create").restype = C.c_int
            f("destroy").argtypes = [C.c_void_p]
            f("destroy").restype = None
            f("push").argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.c_int32, C.POINTER(PushResult)]
            f("push").restype = C.c_int
            f("push_aggregate").argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32, C.POINTER(PushResult)]
            f("push_aggregate").restype = C.c_int
            f("leaf_mean").argtypes = [C.c_void_p, C.c_uint32, C.c_uint64, C.c_void_p]
            f("leaf_mean").restype = None
            f("pull").argtypes = [C.c_void_p, C.c_void_p]
            f("pull").restype = C.c_uint64
            f("gradients_per_update").argtypes = [C.POINTER(_Config)]
            f("gradients_per_update").restype = C.c_uint32
            f("set_alpha0").argtypes = [C.c_void_p, C.c_float]
            f("set_alpha0").restype = C.c_int
            f("norms").argtypes = [C.c_void_p, C.c_void_p]
            f("norms").restype = None
            for n in ("n_updates", "n_pushes", "n_rejected", "sigma_sum", "sigma_max", "hist_len"):
                f(n).argtypes = [C.c_void_p]
                f(n).restype = C.c_uint64
            for n in ("pending", "c", "clock_cap"):
                f(n).argtypes = [C.c_void_p]
                f(n).restype = C.c_uint32
            for n in ("theta", "velocity", "hist", "clocks", "counts", "avg_staleness", "lr_log"):
                f(n).argtypes = [C.c_void_p]
                f(n).restype = C.c_void_p
    return _lib


def gradients_per_update(n_learners, n_split=1, protocol=SOFTSYNC, c_override=0) -> int:
    cfg = _Config(1, n_learners, n_split, c_override, protocol, LR_CONST, 0, 1, 0, 0, OPT_SGD, 0, 0)
    return int(_load().oracle32_gradients_per_update(C.byref(cfg)))


def leaf_mean(grads, precision=32):
    """Average relayed by a tree node: (g_1 + ... + g_k) * (1/k) in arrival order, as binary32."""
    gs = [np.ascontiguousarray(g, dtype=np.float32) for g in grads]
    ptrs = (C.c_void_p * len(gs))(*[g.ctypes.data for g in gs])
    out = np.empty(gs[0].size, np.float32)
    getattr(_load(), ("oracle32_" if precision == 32 else "oracle64_") + "leaf_mean")(ptrs, len(gs), gs[0].size, out.ctypes.data)
    return out


class OracleError(Exception):
    def __init__(self, code):
        super().__init__(f"oracle error {code}")
        self.code = code


class OraclePS:
    """One parameter server replayed on the CPU.  push()/pull() mirror the paper's
    pushGradient / pullWeights messages as the server handles them."""

    def __init__(self, init_weights, n_learners, n_split=1, protocol=SOFTSYNC,
                 lr_mode=LR_AVG_STALENESS, alpha0=0.01, lr_scale=1.0, momentum=0.0,
                 weight_decay=0.0, c_override=0, precision=32, optimizer=OPT_SGD, adagrad_eps=1e-8,
                 max_aggregate=0):
        lib = _load()
        assert precision in (32, 64)
        self._p = "oracle32_" if precision == 32 else "oracle64_"
        self.real = np.float32 if precision == 32 else np.float64
        w = np.ascontiguousarray(init_weights, dtype=np.float32)
        self.n_params = int(w.size)
        self.cfg = _Config(self.n_params, n_learners, n_split, c_override, protocol, lr_mode,
                           alpha0, lr_scale, momentum, weight_decay, optimizer, adagrad_eps, max_aggregate)
        h = C.c_void_p()
        rc = getattr(lib, self._p + "create")(C.byref(self.cfg), w.ctypes.data, C.byref(h))
        if rc != OK:
            raise OracleError(rc)
        self._h = h
        self._lib = lib

    def _f(self, name):
        return getattr(self._lib, self._p + name)

    def close(self):
        if getattr(self, "_h", None):
            self._f("destroy")(self._h)
            self._h = None

    __del__ = close

    def push(self, grad, ts, learner=-1):
        """Returns (rc, PushResult).  rc < 0: rejected, state unchanged."""
        g = np.ascontiguousarray(grad, dtype=np.float32)
        assert g.size == self.n_params
        res = PushResult()
        rc = self._f("push")(self._h, g.ctypes.data, int(ts), int(learner), C.byref(res))
        return rc, res

    def push_aggregate(self, avg, ts_list):
        """A relayed average standing for len(ts_list) learner gradients.  Returns (rc, PushResult)."""
        g = np.ascontiguousarray(avg, dtype=np.float32)
        assert g.size == self.n_params
        ts = np.ascontiguousarray(ts_list, dtype=np.uint64)
        res = PushResult()
        rc = self._f("push_aggregate")(self._h, g.ctypes.data, ts.ctypes.data, int(ts.size), C.byref(res))
        return rc, res

    def pull(self, want_weights=True):
        """(theta as float32 or None, timestamp)."""
        if want_weights:
            dst = np.empty(self.n_params, dtype=np.float32)
            ts = self._f("pull")(self._h, dst.ctypes.data)
            return dst, int(ts)
        return None, int(self._f("pull")(self._h, None))

    def set_alpha0(self, alpha0):
        self._f("set_alpha0")(self._h, alpha0)

    def _array(self, name, n, dtype):
        ptr = self._f(name)(self._h)
        if not ptr or n == 0:
            return np.zeros(0, dtype=dtype)
        buf = (C.c_char * (n * np.dtype(dtype).itemsize)).from_address(ptr)
        return np.frombuffer(buf, dtype=dtype).copy()

    @property
    def theta(self):
        return self._array("theta", self.n_params, self.real)

    @property
    def velocity(self):
        return self._array("velocity", self.n_params, self.real)

    @property
    def ts(self):
        return int(self._f("pull")(self._h, None))

    @property
    def c(self):
        return int(self._f("c")(self._h))

    @property
    def n_updates(self):
        return int(self._f("n_updates")(self._h))

    @property
    def n_pushes(self):
        return int(self._f("n_pushes")(self._h))

    @property
    def n_rejected(self):
        return int(self._f("n_rejected")(self._h))

    @property
    def pending(self):
        return int(self._f("pending")(self._h))

    @property
    def sigma_sum(self):
        return int(self._f("sigma_sum")(self._h))

    @property
    def sigma_max(self):
        return int(self._f("sigma_max")(self._h))

    @property
    def hist(self):
        h = self._array("hist", int(self._f("hist_len")(self._h)), np.uint64)
        nz = np.nonzero(h)[0]
        return h[: (nz[-1] + 1) if nz.size else 0]

    @property
    def clocks(self):
        """Timestamps of the gradients that triggered each update: an (n_updates, c) array, or, when relayed
        averages made some updates collect more than c gradients, a list of arrays."""
        cap = int(self._f("clock_cap")(self._h))
        rows = self._array("clocks", self.n_updates * cap, np.uint64).reshape(self.n_updates, cap)
        counts = self._array("counts", self.n_updates, np.uint32)
        if cap == self.c or (counts == self.c).all():
            return rows[:, :self.c]
        return [rows[u, :counts[u]] for u in range(self.n_updates)]

    @property
    def avg_staleness(self):
        return self._array("avg_staleness", self.n_updates, np.float64)

    @property
    def lr_log(self):
        return self._array("lr_log", self.n_updates, np.float32)

    def norms(self):
        """dict(theta_sq, theta_inf, v_sq, gbar_sq) summed in binary64."""
        out = np.zeros(4, dtype=np.float64)
        self._f("norms")(self._h, out.ctypes.data)
        return dict(theta_sq=out[0], theta_inf=out[1], v_sq=out[2], gbar_sq=out[3])
