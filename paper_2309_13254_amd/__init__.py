"""MI355X-native sparse-gradient encode + aggregate (Zen's Balanced Parallelism hot path).

`binding` is a thin ctypes layer over the C-ABI library built from csrc/ (see include/zen.h); every
step of the path runs in the HIP kernels.  PyTorch is used for device memory and streams only.
"""
from .binding import *  # noqa: F401,F403
from .binding import __all__  # noqa: F401
