"""MI355X-native DP-LLM decode hot path: any-precision GEMV + runtime precision selector.

Thin ctypes binding over libdpllm.so (hand-written HIP for gfx950).  Every step of the path runs
in the library's kernels; this package only marshals pointers.  There is no CPU fallback: if the
library is missing, importing the binding raises.
"""
from .binding import *  # noqa: F401,F403
