"""MI355X-native parameter-server update path of Rudra (arXiv 1509.04210).

The product is the C-ABI HIP library `lib/librudra_ps.so` (declared in include/rudra_ps.h);
this package is its thin ctypes binding.  There is no CPU fallback: importing `binding`
without the built library raises.
"""
from .binding import (  # noqa: F401
    FLAG_CHECK_POINTERS, FLAG_CONTROL_ONLY, FLAG_DOUBLE_BUFFER, FLAG_PUSH_ACCUMULATE, FLAG_STATS_NORMS, FLAG_TIME_KERNELS, HARDSYNC, LR_AVG_STALENESS,
    LR_CONST, LR_PER_GRADIENT, LR_STATIC_N, OPT_ADAGRAD, OPT_SGD, SOFTSYNC, ParameterServer, PushResult, RudraError, Stats, leaf_mean, lib,
    strerror)
