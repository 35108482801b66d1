"""libknapattn for MI355X: packed variable-length joint self-attention (forward
and backward HIP kernels for gfx950) and the host-side workload model and greedy
balancer of KnapFormer.  Thin Python binding over the C ABI in include/knapattn.h.
"""
from .binding import *  # noqa: F401,F403
from .binding import EXPORTS, LIB_PATH, KnapError, lib  # noqa: F401
from .runtime import VarlenAttention  # noqa: F401
