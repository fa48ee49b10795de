"""MI355X (gfx950) library for target-side verification of a draft token tree on a sparse MoE
layer and EVICT's cost-aware prefix selection. The work is done by hand-written HIP kernels
behind a C ABI (include/evict.h, built into libevict.so); this package is the thin ctypes
binding over it. There is no CPU fallback: calls raise if the library is missing."""
from .binding import *  # noqa: F401,F403
