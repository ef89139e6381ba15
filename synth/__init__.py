"""Seeded synthetic inputs (arrival traces, initial weights, gradients) for the
Rudra parameter-server tests and benchmark.  Input generators only: none of the
server's arithmetic lives here, and the generator modules imported below import
neither the CPU oracle nor the HIP library.  `synth.learners` (imported on demand
by the GPU tests, smoke() and bench.py only) is the emulated-learner harness that
feeds these inputs to the HIP library through its ctypes binding."""
from . import configs, gradgen, replay, trace  # noqa: F401
