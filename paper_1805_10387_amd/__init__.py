"""MI355X (gfx950) mixed-precision training step: HIP kernels behind the C ABI of include/mp.h.

`binding` mirrors the C entry points one to one; `steps` strings them into the training
iterations of the five workloads (host control flow only - every computation is a kernel of
libmp.so, and importing this package never falls back to PyTorch or CPU arithmetic)."""
from . import _lib  # noqa: F401
from .binding import *  # noqa: F401,F403
