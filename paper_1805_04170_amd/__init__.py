"""MI355X-native execution of layer chains under k-cut tensor tilings (arXiv 1805.04170).

Thin ctypes binding over libtensor_tiling.so (C ABI in include/tensor_tiling.h).  All computation runs in the
library's HIP kernels; this package only marshals arguments.  PyTorch supplies device memory and streams.
"""
from .binding import *  # noqa: F401,F403
