"""ctypes binding of include/rudra_ps.h: argument marshalling only.

Names follow the C ABI (rudra_ps_create -> ParameterServer(...), rudra_ps_push_gradient ->
.push_gradient, ...).  Device buffers are passed as integer addresses (e.g. torch
`tensor.data_ptr()`); the stream as the integer hipStream_t (torch `stream.cuda_stream`).
"""
from __future__ import annotations

import ctypes as C
import os

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "lib", "librudra_ps.so")

HARDSYNC, SOFTSYNC = 0, 1
LR_CONST, LR_STATIC_N, LR_AVG_STALENESS, LR_PER_GRADIENT = 0, 1, 2, 3
OPT_SGD, OPT_ADAGRAD = 0, 1
FLAG_STATS_NORMS, FLAG_PUSH_ACCUMULATE, FLAG_CONTROL_ONLY, FLAG_TIME_KERNELS, FLAG_DOUBLE_BUFFER = 1, 2, 4, 8, 16
FLAG_CHECK_POINTERS = 32
OK, EINVAL, EFUTURE_TS, EHARDSYNC_STALE, EHARDSYNC_DUP, ENOMEM, EHIP, ERANGE, ESTATE = 0, -1, -2, -3, -4, -5, -6, -7, -8


class Config(C.Structure):
    _fields_ = [("n_params", C.c_uint64), ("n_learners", C.c_uint32), ("n_split", C.c_uint32),
                ("c_override", C.c_uint32), ("protocol", C.c_int32), ("lr_mode", C.c_int32),
                ("alpha0", C.c_float), ("lr_scale", C.c_float), ("momentum", C.c_float),
                ("weight_decay", C.c_float), ("optimizer", C.c_int32), ("adagrad_eps", C.c_float), ("device", C.c_int32), ("flags", C.c_uint32),
                ("stream", C.c_void_p), ("clock_ring", C.c_uint32), ("launch_block", C.c_uint32),
                ("launch_unroll", C.c_uint32), ("launch_vec", C.c_uint32), ("launch_grid", C.c_uint32),
                ("launch_waves_per_cu", C.c_uint32), ("max_aggregate", C.c_uint32), ("launch_alternate", C.c_uint32),
                ("launch_state_loads", C.c_uint32), ("launch_phased", C.c_uint32)]


class PushResult(C.Structure):
    _fields_ = [("staleness", C.c_uint64), ("ts_after", C.c_uint64), ("pending", C.c_uint32),
                ("applied", C.c_int32), ("lr_used", C.c_float)]


class Stats(C.Structure):
    _fields_ = [("ts_cur", C.c_uint64), ("n_pushes", C.c_uint64), ("n_updates", C.c_uint64),
                ("n_rejected", C.c_uint64), ("sigma_sum", C.c_uint64), ("sigma_max", C.c_uint64),
                ("hist_len", C.c_uint64), ("bytes_absorbed", C.c_uint64), ("sigma_mean", C.c_double),
                ("last_avg_staleness", C.c_double), ("theta_sq", C.c_double), ("theta_inf", C.c_double),
                ("v_sq", C.c_double), ("gbar_sq", C.c_double), ("kernel_ms", C.c_double),
                ("kernel_launches", C.c_uint64), ("pending", C.c_uint32), ("c", C.c_uint32),
                ("last_lr", C.c_float), ("norms_valid", C.c_int32), ("last_hip_error", C.c_int32),
                ("reserved", C.c_uint32), ("n_weight_copies", C.c_uint64), ("n_ts_inquiries", C.c_uint64),
                ("n_weight_views", C.c_uint64), ("n_apply_launches", C.c_uint64), ("n_batched_updates", C.c_uint64),
                ("n_weight_acquires", C.c_uint64), ("n_reader_waits", C.c_uint64), ("n_phased_launches", C.c_uint64)]


_lib = None


def lib():
    """The loaded HIP library.  Fails loudly when it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()'). "
                               "There is no CPU fallback.")
        L = C.CDLL(LIB_PATH)
        vp, u64, u32, i32 = C.c_void_p, C.c_uint64, C.c_uint32, C.c_int32
        sigs = {
            "rudra_ps_create": [C.POINTER(Config), vp, C.POINTER(vp)],
            "rudra_ps_destroy": [vp],
            "rudra_ps_push_gradient": [vp, vp, u64, i32, C.POINTER(PushResult)],
            "rudra_ps_push_batch": [vp, C.POINTER(vp), C.POINTER(u64), C.POINTER(i32), u32, C.POINTER(PushResult),
                                    C.POINTER(u32)],
            "rudra_ps_push_aggregate": [vp, vp, C.POINTER(u64), u32, C.POINTER(PushResult)],
            "rudra_ps_leaf_mean": [C.POINTER(vp), u32, u64, vp, i32, vp],
            "rudra_ps_pull_weights": [vp, vp, C.POINTER(u64)],
            "rudra_ps_weights_view": [vp, C.POINTER(vp), C.POINTER(u64)],
            "rudra_ps_weights_acquire": [vp, vp, C.POINTER(vp), C.POINTER(u64), C.POINTER(u64)],
            "rudra_ps_weights_release": [vp, u64, vp],
            "rudra_ps_pull_weights_on": [vp, vp, vp, C.POINTER(u64)],
            "rudra_ps_broadcast_weights": [vp, C.POINTER(vp), u32, vp, C.POINTER(u64)],
            "rudra_ps_launch_shape": [vp, i32, C.POINTER(u32), C.POINTER(u32), C.POINTER(u64), C.POINTER(u32)],
            "rudra_ps_pull_velocity": [vp, vp],
            "rudra_ps_stats": [vp, C.POINTER(Stats)],
            "rudra_ps_staleness_hist": [vp, C.POINTER(u64), u64, C.POINTER(u64)],
            "rudra_ps_vector_clock": [vp, u64, C.POINTER(u64), u32, C.POINTER(u32), C.POINTER(C.c_double),
                                      C.POINTER(C.c_float)],
            "rudra_ps_set_lr": [vp, C.c_float],
            "rudra_ps_sync": [vp],
        }
        sigs["rudra_ps_apply_update_noalloc"] = [C.POINTER(vp), u32, u64, vp, vp, C.c_float, C.c_float, C.c_float, i32, C.c_float,
                                                 vp, i32, vp]
        for name, args in sigs.items():
            fn = getattr(L, name)
            fn.argtypes, fn.restype = args, C.c_int
        L.rudra_ps_strerror.argtypes, L.rudra_ps_strerror.restype = [C.c_int], C.c_char_p
        _lib = L
    return _lib


def strerror(status: int) -> str:
    return lib().rudra_ps_strerror(status).decode()


class RudraError(RuntimeError):
    def __init__(self, status, what):
        super().__init__(f"{what}: {strerror(status)} ({status})")
        self.status = status


def leaf_mean(grad_ptrs, n_params, out_ptr, device=0, stream=0):
    """rudra_ps_leaf_mean: out = (g_1 + ... + g_k) * (1/k) on the device."""
    arr = (C.c_void_p * len(grad_ptrs))(*grad_ptrs)
    rc = lib().rudra_ps_leaf_mean(arr, len(grad_ptrs), n_params, out_ptr, device, stream or None)
    if rc != OK:
        raise RudraError(rc, "rudra_ps_leaf_mean")


def apply_update_noalloc(grad_ptrs, n_params, theta_ptr, state_ptr, lr, momentum=0.0, weight_decay=0.0, optimizer=OPT_SGD,
                         adagrad_eps=1e-8, norms_out_ptr=0, device=0, stream=0):
    """rudra_ps_apply_update_noalloc: returns the C status."""
    arr = (C.c_void_p * max(1, len(grad_ptrs)))(*grad_ptrs)
    return lib().rudra_ps_apply_update_noalloc(arr, len(grad_ptrs), n_params, theta_ptr or None, state_ptr or None, lr, momentum,
                                               weight_decay, optimizer, adagrad_eps, norms_out_ptr or None, device, stream or None)


class ParameterServer:
    """One rudra_ps_t.  Methods return the C status where a caller may want to see a rejection
    (push_gradient) and raise RudraError otherwise."""

    def __init__(self, n_params, n_learners, init_weights_ptr=0, n_split=1, protocol=SOFTSYNC,
                 lr_mode=LR_AVG_STALENESS, alpha0=0.01, lr_scale=1.0, momentum=0.0, weight_decay=0.0,
                 c_override=0, device=0, stream=0, flags=0, clock_ring=0, launch_block=0, launch_unroll=0,
                 launch_vec=0, launch_grid=0, launch_waves_per_cu=0, launch_alternate=0, optimizer=OPT_SGD,
                 adagrad_eps=1e-8, max_aggregate=0, launch_state_loads=0, launch_phased=0):
        self._L = lib()
        self.cfg = Config(n_params, n_learners, n_split, c_override, protocol, lr_mode, alpha0, lr_scale, momentum,
                          weight_decay, optimizer, adagrad_eps, device, flags, stream or None, clock_ring, launch_block, launch_unroll,
                          launch_vec, launch_grid, launch_waves_per_cu, max_aggregate, launch_alternate, launch_state_loads, launch_phased)
        h = C.c_void_p()
        rc = self._L.rudra_ps_create(C.byref(self.cfg), init_weights_ptr or None, C.byref(h))
        if rc != OK:
            raise RudraError(rc, "rudra_ps_create")
        self._h = h
        self.n_params = n_params
        self._res = PushResult()
        self._res_ref = C.byref(self._res)
        self._push = self._L.rudra_ps_push_gradient

    def destroy(self):
        if getattr(self, "_h", None):
            self._L.rudra_ps_destroy(self._h)
            self._h = None

    __del__ = destroy

    def push_gradient(self, grad_ptr, ts, learner=-1):
        """(status, PushResult).  The PushResult object is reused by the next call."""
        return self._push(self._h, grad_ptr or None, ts, learner, self._res_ref), self._res

    def push_batch(self, grad_ptrs, ts_list, learners=None):
        """rudra_ps_push_batch: a run of messages in one call.  (status, n_handled, [PushResult] * n_handled)."""
        n = len(ts_list)
        ptrs = (C.c_void_p * n)(*[p or None for p in grad_ptrs])
        ts = (C.c_uint64 * n)(*ts_list)
        ls = (C.c_int32 * n)(*learners) if learners is not None else None
        res = (PushResult * n)()
        handled = C.c_uint32()
        rc = self._L.rudra_ps_push_batch(self._h, ptrs, ts, ls, n, res, C.byref(handled))
        return rc, handled.value, res[:handled.value]

    def push_aggregate(self, avg_ptr, ts_list):
        """A relayed average standing for len(ts_list) learner gradients.  (status, PushResult)."""
        ts = (C.c_uint64 * len(ts_list))(*ts_list)
        rc = self._L.rudra_ps_push_aggregate(self._h, avg_ptr or None, ts, len(ts_list), C.byref(self._res))
        return rc, self._res

    def pull_weights(self, dst_ptr=0):
        """Timestamp of the weights; with dst_ptr also enqueues the copy of theta."""
        ts = C.c_uint64()
        rc = self._L.rudra_ps_pull_weights(self._h, dst_ptr or None, C.byref(ts))
        if rc != OK:
            raise RudraError(rc, "rudra_ps_pull_weights")
        return ts.value

    def pull_weights_on(self, dst_ptr, reader_stream=0):
        """Timestamp of the weights; the copy into dst_ptr runs on reader_stream, ordered against the server's launches."""
        ts = C.c_uint64()
        rc = self._L.rudra_ps_pull_weights_on(self._h, dst_ptr, reader_stream or None, C.byref(ts))
        if rc != OK:
            raise RudraError(rc, "rudra_ps_pull_weights_on")
        return ts.value

    def broadcast_weights(self, dst_ptrs, reader_stream=0):
        """Timestamp of the weights; one launch on reader_stream writes them to every address in dst_ptrs."""
        k = len(dst_ptrs)
        arr = (C.c_void_p * k)(*dst_ptrs)
        ts = C.c_uint64()
        rc = self._L.rudra_ps_broadcast_weights(self._h, arr, k, reader_stream or None, C.byref(ts))
        if rc != OK:
            raise RudraError(rc, "rudra_ps_broadcast_weights")
        return ts.value

    def weights_view(self):
        """(device address of the current weights, their timestamp): zero-copy pullWeights."""
        p, ts = C.c_void_p(), C.c_uint64()
        rc = self._L.rudra_ps_weights_view(self._h, C.byref(p), C.byref(ts))
        if rc != OK:
            raise RudraError(rc, "rudra_ps_weights_view")
        return p.value, ts.value

    def weights_acquire(self, reader_stream=0):
        """(device address of the current weights, their timestamp, ticket) for reads enqueued on `reader_stream`."""
        p, ts, ticket = C.c_void_p(), C.c_uint64(), C.c_uint64()
        rc = self._L.rudra_ps_weights_acquire(self._h, reader_stream or None, C.byref(p), C.byref(ts), C.byref(ticket))
        if rc != OK:
            raise RudraError(rc, "rudra_ps_weights_acquire")
        return p.value, ts.value, ticket.value

    def weights_release(self, ticket, reader_stream=0):
        """The C status: OK, or ESTATE when the buffer's overwriting launch was already enqueued."""
        return self._L.rudra_ps_weights_release(self._h, ticket, reader_stream or None)

    def launch_shape(self, batched=False):
        """(grid, block, ntiles, lds_bytes) of the next single-update or batched launch."""
        g, b, t, l = C.c_uint32(), C.c_uint32(), C.c_uint64(), C.c_uint32()
        rc = self._L.rudra_ps_launch_shape(self._h, int(batched), C.byref(g), C.byref(b), C.byref(t), C.byref(l))
        if rc != OK:
            raise RudraError(rc, "rudra_ps_launch_shape")
        return g.value, b.value, t.value, l.value

    def pull_velocity(self, dst_ptr):
        rc = self._L.rudra_ps_pull_velocity(self._h, dst_ptr)
        if rc != OK:
            raise RudraError(rc, "rudra_ps_pull_velocity")

    def stats(self) -> Stats:
        st = Stats()
        rc = self._L.rudra_ps_stats(self._h, C.byref(st))
        if rc != OK:
            raise RudraError(rc, "rudra_ps_stats")
        return st

    def staleness_hist(self):
        n = C.c_uint64()
        self._L.rudra_ps_staleness_hist(self._h, None, 0, C.byref(n))
        buf = (C.c_uint64 * max(1, n.value))()
        rc = self._L.rudra_ps_staleness_hist(self._h, buf, n.value, C.byref(n))
        if rc != OK:
            raise RudraError(rc, "rudra_ps_staleness_hist")
        return list(buf[:n.value])

    def vector_clock(self, update_idx):
        """(timestamps, <sigma>, lr) of one update; raises RudraError(ERANGE) if it left the ring."""
        cap = self.stats().c + self.cfg.max_aggregate       # an update collects at most c + max_aggregate - 1 gradients
        buf = (C.c_uint64 * cap)()
        n, avg, lr = C.c_uint32(), C.c_double(), C.c_float()
        rc = self._L.rudra_ps_vector_clock(self._h, update_idx, buf, cap, C.byref(n), C.byref(avg), C.byref(lr))
        if rc != OK:
            raise RudraError(rc, "rudra_ps_vector_clock")
        return list(buf[:n.value]), avg.value, lr.value

    def set_lr(self, alpha0):
        rc = self._L.rudra_ps_set_lr(self._h, alpha0)
        if rc != OK:
            raise RudraError(rc, "rudra_ps_set_lr")

    def sync(self):
        rc = self._L.rudra_ps_sync(self._h)
        if rc != OK:
            raise RudraError(rc, "rudra_ps_sync")
