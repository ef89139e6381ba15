"""Seeded synthetic inputs (arrival traces, initial weights, gradients) for the
Rudra parameter-server tests and benchmark.  Input generators only: none of the
server's arithmetic lives here, and this package imports neither the CPU oracle
nor the HIP library."""
from . import configs, gradgen, replay, trace  # noqa: F401
