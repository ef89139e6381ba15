"""The emulated learners' loop: plumbing shared by every server under test.

`server` is anything with
    push(learner, step, ts) -> (rc, staleness, applied)   # pushGradient of that learner's step-th gradient
    pull_ts() -> int                                      # timestamp inquiry of pullWeights
How the gradient of (learner, step) is materialised (host array for the oracle,
device buffer for the HIP library) is the adapter's business.

Learner behaviour (Sec. 3.2 "Learner"): it pulls the weights and their timestamp
before each mini-batch and stamps the gradient with that timestamp.  Here the
pull happens right after the learner's previous push was handled (zero
communication time); under hardsync every learner re-pulls after the update
(the server broadcasts the new weights).
"""
from __future__ import annotations

import numpy as np


def replay(server, learner, step, n_learners, hardsync=False):
    """Drive `server` through the arrival trace.  Returns a log dict of int64 arrays:
    ts_pushed, ts_at_arrival, staleness, applied (one entry per push)."""
    n = len(learner)
    learner_ts = np.zeros(n_learners, dtype=np.int64)  # all learners start from the weights stamped 0
    log = dict(ts_pushed=np.zeros(n, np.int64), ts_at_arrival=np.zeros(n, np.int64),
               staleness=np.zeros(n, np.int64), applied=np.zeros(n, np.int64))
    for i in range(n):
        l, s = int(learner[i]), int(step[i])
        ts = int(learner_ts[l])
        log["ts_at_arrival"][i] = server.pull_ts()
        rc, sigma, applied = server.push(l, s, ts)
        if rc != 0:
            raise RuntimeError(f"push {i} (learner {l}, step {s}, ts {ts}) rejected: {rc}")
        log["ts_pushed"][i] = ts
        log["staleness"][i] = sigma
        log["applied"][i] = applied
        now = server.pull_ts()
        if hardsync and applied:
            learner_ts[:] = now
        else:
            learner_ts[l] = now
    return log
