"""Adapter that lets the emulated-learner loop (synth.replay) drive the CPU oracle.
TEST INFRASTRUCTURE, like everything under oracle/."""
from __future__ import annotations

import numpy as np

from . import leaf_mean
from . import (HARDSYNC, LR_AVG_STALENESS, LR_CONST, LR_PER_GRADIENT, LR_STATIC_N, OPT_ADAGRAD, OPT_SGD, SOFTSYNC,
               OraclePS)

PROTOCOL = {"hardsync": HARDSYNC, "softsync": SOFTSYNC}
LR_MODE = {"const": LR_CONST, "static_n": LR_STATIC_N, "avg_staleness": LR_AVG_STALENESS,
           "per_gradient": LR_PER_GRADIENT}
OPTIMIZER = {"sgd": OPT_SGD, "adagrad": OPT_ADAGRAD}


class OracleServer:
    """Oracle over the elements `index` of a workload's parameter vector (default: all of
    them).  The update is elementwise, so a subset of indices replays exactly what the
    full vector would hold at those positions."""

    def __init__(self, workload, index=None, precision=32, max_aggregate=0):
        self.w = workload
        self.index = np.arange(workload.n_params, dtype=np.uint64) if index is None else np.asarray(index, np.uint64)
        self.ps = OraclePS(workload.init_weights_at(self.index), workload.n_learners, workload.n_split,
                           PROTOCOL[workload.protocol], LR_MODE[workload.lr_mode], workload.alpha0,
                           workload.lr_scale, workload.momentum, workload.weight_decay, workload.c_override,
                           precision=precision, optimizer=OPTIMIZER[workload.optimizer],
                           adagrad_eps=workload.adagrad_eps, max_aggregate=max_aggregate)
        self.precision = precision

    def push(self, learner, step, ts):
        rc, res = self.ps.push(self.w.grad_at(learner, step, self.index), ts, learner)
        return rc, int(res.staleness), int(res.applied)

    def push_batch(self, messages):
        """A run of messages: the oracle knows no batches, it takes them one by one."""
        sigma, applied = [], []
        for i, (l, s, ts) in enumerate(messages):
            rc, sg, ap = self.push(l, s, ts)
            if rc != 0:
                return rc, i, sigma, applied
            sigma.append(sg)
            applied.append(ap)
        return 0, len(messages), sigma, applied

    def push_aggregate(self, members, ts_list):
        """What a tree node relays for `members` = [(learner, step), ...]: their average, with their timestamps."""
        avg = leaf_mean([self.w.grad_at(l, s, self.index) for l, s in members], self.precision)
        rc, res = self.ps.push_aggregate(avg, ts_list)
        return rc, int(res.staleness), int(res.applied)

    def pull_ts(self):
        return self.ps.ts
