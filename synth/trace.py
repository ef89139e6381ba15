"""Seeded arrival traces: lambda emulated learners as a discrete-event simulation.

INPUT generator only.  A trace is the ORDER in which learners' pushGradient
messages reach the server: a list of (learner, step) pairs, `step` counting that
learner's own mini-batches.  It contains no timestamps: the timestamp a learner
attaches to a gradient is the one it got from its latest pullWeights (Sec. 3.2
"Learner"), which the replay loop obtains from whichever server it is driving.

Softsync: learner l finishes its s-th mini-batch at T_l(s) = sum_{j<=s} d(l, j),
d ~ Exp(1) (times a straggler factor with the stated probability), zero
communication time; the server sees the pushes merged by finish time (ties ->
lower learner id).  Hardsync: rounds; in round r every learner computes one
mini-batch and the lambda pushes arrive in order of their Exp(1) durations.
"""
from __future__ import annotations

import heapq
import math

import numpy as np

from .gradgen import TAG_STRAGGLER, TAG_TIME, uniform01


def _duration(seed, learner, step, straggler_prob, straggler_factor, jitter):
    u = uniform01(seed, TAG_TIME, learner, step)
    if jitter is not None:  # near-homogeneous cluster: 1 +- jitter, uniform
        d = 1.0 + jitter * (2.0 * u - 1.0)
    else:
        d = -math.log(u)  # Exp(1)
    if straggler_prob > 0.0 and uniform01(seed, TAG_STRAGGLER, learner, step) <= straggler_prob:
        d *= straggler_factor
    return d


def softsync_trace(seed, n_learners, n_pushes, straggler_prob=0.0, straggler_factor=3.0, jitter=None):
    """(learner[int32], step[int32]) arrays of length n_pushes."""
    heap = []
    for l in range(n_learners):
        heapq.heappush(heap, (_duration(seed, l, 0, straggler_prob, straggler_factor, jitter), l, 0))
    learner = np.empty(n_pushes, dtype=np.int32)
    step = np.empty(n_pushes, dtype=np.int32)
    for i in range(n_pushes):
        t, l, s = heapq.heappop(heap)
        learner[i], step[i] = l, s
        heapq.heappush(heap, (t + _duration(seed, l, s + 1, straggler_prob, straggler_factor, jitter), l, s + 1))
    return learner, step


def hardsync_trace(seed, n_learners, n_rounds, straggler_prob=0.0, straggler_factor=3.0):
    learner = np.empty(n_rounds * n_learners, dtype=np.int32)
    step = np.empty(n_rounds * n_learners, dtype=np.int32)
    for r in range(n_rounds):
        order = sorted(range(n_learners),
                       key=lambda l: (_duration(seed, l, r, straggler_prob, straggler_factor, None), l))
        learner[r * n_learners:(r + 1) * n_learners] = order
        step[r * n_learners:(r + 1) * n_learners] = r
    return learner, step
