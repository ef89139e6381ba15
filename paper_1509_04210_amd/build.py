"""Builds the HIP shared library for gfx950 with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess

_PKG = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_PKG)
SRC = os.path.join(_PKG, "csrc", "rudra_ps.hip")
HEADERS = [os.path.join(_PKG, "csrc", "apply_update.hip.h"), os.path.join(_ROOT, "include", "rudra_ps.h")]
LIB = os.path.join(_PKG, "lib", "librudra_ps.so")

# -ffp-contract=off: every fp32 operation of the update rule is rounded on its own (bit parity with a
# sequential evaluation).  packed-fp32 ops are switched off for the test machines.
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off",
               "-fno-fast-math", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-Wall", "-Wno-unused-command-line-argument"]


def build(force: bool = True, extra_flags=(), out: str | None = None) -> str:
    out = out or LIB
    if not force and os.path.exists(out) and all(os.path.getmtime(out) >= os.path.getmtime(f) for f in [SRC, *HEADERS]):
        return out
    os.makedirs(os.path.dirname(out), exist_ok=True)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    subprocess.run([hipcc, *HIPCC_FLAGS, *extra_flags, SRC, "-o", out], check=True)
    return out


if __name__ == "__main__":
    print(build())
