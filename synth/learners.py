"""Emulated learners feeding one ParameterServer on one GPU.

Harness used by the GPU tests, smoke() and bench.py (not part of the library's package): torch
supplies device memory and the stream, synth supplies the seeded gradients (generated on the
device) and the arrival trace, and every step of the update path itself runs inside the HIP
library, reached through its ctypes binding.  Holds none of the method's arithmetic.
"""
from __future__ import annotations

import torch

from paper_1509_04210_amd import binding as B

from . import gradgen

PROTOCOL = {"hardsync": B.HARDSYNC, "softsync": B.SOFTSYNC}
LR_MODE = {"const": B.LR_CONST, "static_n": B.LR_STATIC_N, "avg_staleness": B.LR_AVG_STALENESS,
           "per_gradient": B.LR_PER_GRADIENT}
OPTIMIZER = {"sgd": B.OPT_SGD, "adagrad": B.OPT_ADAGRAD}


class HipServer:
    """A workload's parameter server on `device`, plus a ring of gradient buffers.

    push(learner, step, ts) materialises that learner's gradient into the next ring buffer (generator kernel
    on the server's stream) and pushes it.  With `pregenerated` > 0 the ring is filled once with that many
    distinct gradients and pushes cycle through it without generating (throughput runs).
    The ring holds at least c+1 buffers, so a buffer is only rewritten after the update that
    consumed it was enqueued on the same stream.
    """

    def __init__(self, workload, flags=0, device=0, ring=None, pregenerated=0, avg_ring=0, **launch):
        self.w = workload
        self.dev = torch.device("cuda", device)
        self.stream = torch.cuda.Stream(device=self.dev)
        P = workload.n_params
        n_ring = max(ring or 0, pregenerated, workload.c + 1)
        self.ring = [torch.empty(P, dtype=torch.float32, device=self.dev) for _ in range(n_ring)]
        init = torch.empty(P, dtype=torch.float32, device=self.dev)
        torch.cuda.synchronize(self.dev)
        self.sh = self.stream.cuda_stream
        gradgen.fill_device(init.data_ptr(), P, workload.init_key(), workload.init_std, stream=self.sh)
        self.ps = B.ParameterServer(P, workload.n_learners, init.data_ptr(), workload.n_split,
                                    PROTOCOL[workload.protocol], LR_MODE[workload.lr_mode], workload.alpha0,
                                    workload.lr_scale, workload.momentum, workload.weight_decay,
                                    workload.c_override, device, self.sh, flags, optimizer=OPTIMIZER[workload.optimizer],
                                    adagrad_eps=workload.adagrad_eps, **launch)
        # tree mode: buffers for relayed averages (borrowed by the root until its update has run)
        self.avg_ring = [torch.empty(P, dtype=torch.float32, device=self.dev) for _ in range(avg_ring)]
        self._next_avg = 0
        self.pregenerated = pregenerated
        for i in range(pregenerated):
            self._fill(self.ring[i], i % workload.n_learners, i // workload.n_learners)
        self.ps.sync()
        del init
        self._next = 0

    def _fill(self, buf, learner, step):
        w = self.w
        gradgen.fill_device(buf.data_ptr(), w.n_params, w.grad_key(learner, step), w.grad_std, w.tail_per,
                            w.tail_factor, stream=self.sh)

    def push(self, learner, step, ts):
        buf = self.ring[self._next]
        self._next = (self._next + 1) % (self.pregenerated or len(self.ring))
        if not self.pregenerated:
            self._fill(buf, learner, step)
        rc, res = self.ps.push_gradient(buf.data_ptr(), ts, learner)
        return rc, res.staleness, res.applied

    def push_batch(self, messages):
        """rudra_ps_push_batch for `messages` = [(learner, step, ts), ...]: every gradient is materialised into its own
        ring buffer first (the ring must hold the batch plus whatever was pending before it)."""
        assert len(messages) + self.w.c <= len(self.ring) or self.pregenerated, "ring too small for this batch"
        ptrs = []
        for l, s, _ in messages:
            buf = self.ring[self._next]
            self._next = (self._next + 1) % (self.pregenerated or len(self.ring))
            if not self.pregenerated:
                self._fill(buf, l, s)
            ptrs.append(buf.data_ptr())
        rc, handled, res = self.ps.push_batch(ptrs, [ts for _, _, ts in messages], [l for l, _, _ in messages])
        return rc, handled, [r.staleness for r in res], [r.applied for r in res]

    def push_aggregate(self, members, ts_list):
        """A tree node's work for `members` = [(learner, step), ...]: materialise their gradients, average them on the
        device (rudra_ps_leaf_mean) and relay the average with the members' timestamps to the root."""
        ptrs = []
        for l, s in members:
            buf = self.ring[self._next]
            self._next = (self._next + 1) % len(self.ring)
            self._fill(buf, l, s)
            ptrs.append(buf.data_ptr())
        avg = self.avg_ring[self._next_avg]
        self._next_avg = (self._next_avg + 1) % len(self.avg_ring)
        B.leaf_mean(ptrs, self.w.n_params, avg.data_ptr(), self.dev.index or 0, self.sh)
        rc, res = self.ps.push_aggregate(avg.data_ptr(), ts_list)
        return rc, res.staleness, res.applied

    def pull_ts(self):
        return self.ps.pull_weights(0)

    def weights(self):
        out = torch.empty(self.w.n_params, dtype=torch.float32, device=self.dev)
        torch.cuda.synchronize(self.dev)
        self.ps.pull_weights(out.data_ptr())
        self.ps.sync()
        return out

    def velocity(self):
        out = torch.empty(self.w.n_params, dtype=torch.float32, device=self.dev)
        torch.cuda.synchronize(self.dev)
        self.ps.pull_velocity(out.data_ptr())
        self.ps.sync()
        return out

    def close(self):
        self.ps.destroy()
        self.ring = []
