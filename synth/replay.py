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


def replay_tree(server, learner, step, n_learners, fan_in, hardsync=False):
    """The same learners under a two-level server tree (Sec. 3.3): learner l talks to node l // fan_in; a node relays
    the average of every `fan_in` gradients it has received (in arrival order) to the root.  `server` needs
        push_aggregate(members, ts_list) -> (rc, staleness, applied)      # members: [(learner, step), ...]
        pull_ts() -> int
    A learner pulls right after handing its gradient to its node (weights travel down the tree at no cost here).
    Returns per-message logs (one entry per relayed average) and what was left waiting in the nodes."""
    n_nodes = -(-n_learners // fan_in)
    waiting = [[] for _ in range(n_nodes)]
    learner_ts = np.zeros(n_learners, dtype=np.int64)
    log = dict(staleness=[], applied=[], ts_at_arrival=[], size=[])
    for i in range(len(learner)):
        l, s = int(learner[i]), int(step[i])
        node = waiting[l // fan_in]
        node.append((l, s, int(learner_ts[l])))
        if len(node) == fan_in:
            log["ts_at_arrival"].append(server.pull_ts())
            rc, sigma, applied = server.push_aggregate([(a, b) for a, b, _ in node], [t for _, _, t in node])
            if rc != 0:
                raise RuntimeError(f"relayed message at push {i} rejected: {rc}")
            log["staleness"].append(sigma)
            log["applied"].append(applied)
            log["size"].append(fan_in)
            node.clear()
            if hardsync and applied:
                learner_ts[:] = server.pull_ts()      # the new weights are broadcast to every learner
        learner_ts[l] = server.pull_ts()
    out = {k: np.array(v, dtype=np.int64) for k, v in log.items()}
    out["left_in_nodes"] = sum(len(n) for n in waiting)
    return out


def replay_batched(server, learner, step, n_learners, chunk_sizes, hardsync=False, c=1):
    """The same learners when the server takes the messages that have queued up in one call: the trace is cut into
    chunks of the given sizes (cycled), and each chunk is one
        push_batch(messages) -> (rc, n_handled, staleness list, applied list)     # messages: [(learner, step, ts), ...]
    A learner stamps its gradient with the timestamp of its last pull and pulls again only after the chunk that held
    its push was handled (a learner appearing twice in a chunk sends both gradients with the same stamp).  Under
    hardsync the stamp must equal the server's timestamp at arrival, which is the number of completed rounds.
    Returns the same log as replay(), minus ts_at_arrival."""
    n = len(learner)
    learner_ts = np.zeros(n_learners, dtype=np.int64)
    log = dict(ts_pushed=np.zeros(n, np.int64), staleness=np.zeros(n, np.int64), applied=np.zeros(n, np.int64))
    i, k = 0, 0
    while i < n:
        m = min(int(chunk_sizes[k % len(chunk_sizes)]), n - i)
        k += 1
        msgs = []
        for j in range(i, i + m):
            l = int(learner[j])
            ts = j // c if hardsync else int(learner_ts[l])
            msgs.append((l, int(step[j]), ts))
            log["ts_pushed"][j] = ts
        rc, handled, sigma, applied = server.push_batch(msgs)
        if rc != 0 or handled != m:
            raise RuntimeError(f"batch at push {i} stopped after {handled} of {m} messages: {rc}")
        log["staleness"][i:i + m] = sigma
        log["applied"][i:i + m] = applied
        now = server.pull_ts()
        for l, _, _ in msgs:
            learner_ts[l] = now
        i += m
    return log
