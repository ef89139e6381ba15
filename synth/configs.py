"""The synthetic workloads (stand-ins for the paper's CIFAR10 / ImageNet runs).

Only vector sizes, learner counts, protocols and hyper-parameters come from the
paper (Sec. 4.2, Sec. 5, Table 4); the numbers flowing through are seeded noise
from gradgen.py.  Protocol and rate mode are plain strings here so that this
module depends on neither the oracle nor the HIP library.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

from . import gradgen, trace


@dataclass(frozen=True)
class Workload:
    name: str
    n_params: int
    n_learners: int            # lambda
    protocol: str              # "hardsync" | "softsync"
    n_split: int               # n of n-softsync (1 under hardsync)
    lr_mode: str               # "const" | "static_n" | "avg_staleness" | "per_gradient"
    alpha0: float
    momentum: float
    weight_decay: float
    n_pushes: int
    grad_std: float
    seed: int
    init_std: float = 0.01
    tail_per: int = 0          # 1/tail_per of the entries scaled by tail_factor (0 = none)
    tail_factor: float = 100.0
    straggler_prob: float = 0.0
    straggler_factor: float = 3.0
    lr_scale: float = 1.0
    c_override: int = 0
    optimizer: str = "sgd"       # "sgd" (momentum optional) | "adagrad"
    adagrad_eps: float = 1e-8

    @property
    def c(self) -> int:
        if self.c_override:
            return self.c_override
        return self.n_learners if self.protocol == "hardsync" else self.n_learners // self.n_split

    def arrival_trace(self, n_pushes=None):
        n = self.n_pushes if n_pushes is None else n_pushes
        if self.protocol == "hardsync":
            rounds = -(-n // self.n_learners)
            l, s = trace.hardsync_trace(self.seed, self.n_learners, rounds, self.straggler_prob, self.straggler_factor)
            return l[:n], s[:n]
        return trace.softsync_trace(self.seed, self.n_learners, n, self.straggler_prob, self.straggler_factor)

    def init_key(self) -> int:
        return gradgen.stream_key(self.seed, gradgen.TAG_INIT)

    def grad_key(self, learner: int, step: int) -> int:
        return gradgen.stream_key(self.seed, gradgen.TAG_GRAD, int(learner), int(step))

    def init_weights_at(self, index):
        return gradgen.values_at(self.init_key(), index, self.init_std)

    def grad_at(self, learner, step, index):
        return gradgen.values_at(self.grad_key(learner, step), index, self.grad_std, self.tail_per, self.tail_factor)

    def scaled(self, n_params=None, n_pushes=None, name=None):
        """Same recipe at another size (parity cases that must finish in seconds on the CPU)."""
        return replace(self, n_params=n_params or self.n_params, n_pushes=n_pushes or self.n_pushes,
                       name=name or self.name)


SEED0 = 0x5EED0000

C1 = Workload("C1-tiny-1softsync", 131072, 4, "softsync", 1, "const", 0.01, 0.0, 0.0, 256, 1e-3, SEED0 + 1)
C2 = Workload("C2-cifar-hardsync", 1_000_000, 30, "hardsync", 1, "const", 0.001, 0.9, 0.0, 30_000, 1e-3, SEED0 + 2)


def C3(n_split: int) -> Workload:
    return Workload(f"C3-cifar-{n_split}softsync", 1_000_000, 30, "softsync", n_split, "avg_staleness", 0.001,
                    0.0, 0.0, 2000, 1e-3, SEED0 + 3, straggler_prob=0.1, straggler_factor=3.0)


C4 = Workload("C4-imagenet-1softsync", 72_000_000, 18, "softsync", 1, "avg_staleness", 0.01, 0.9, 0.0, 3600,
              1e-4, SEED0 + 4, tail_per=100, tail_factor=100.0)
C5 = Workload("C5-imagenet-lambda-softsync", 72_000_000, 54, "softsync", 54, "avg_staleness", 0.01, 0.9, 5e-4,
              5000, 1e-4, SEED0 + 5)

# The paper's ImageNet 1-softsync runs used AdaGrad instead of momentum SGD (Sec. 5.5)
C4_ADAGRAD = Workload("C4-imagenet-1softsync-adagrad", 72_000_000, 18, "softsync", 1, "avg_staleness", 0.01, 0.0, 0.0,
                      3600, 1e-4, SEED0 + 6, tail_per=100, tail_factor=100.0, optimizer="adagrad")

# The 4-softsync case with 8 gradients per update instead of floor(30/4) = 7 (Eq. 5 prints the floor; a rounded
# lambda/n is the other way to read "about 8")
C3_N4_C8 = replace(C3(4), name="C3-cifar-4softsync-c8", c_override=8)

ALL = {"C1": C1, "C2": C2, "C3-n1": C3(1), "C3-n2": C3(2), "C3-n4": C3(4), "C3-n4-c8": C3_N4_C8, "C3-n30": C3(30), "C4": C4,
       "C5": C5, "C4-adagrad": C4_ADAGRAD}
