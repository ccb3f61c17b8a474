"""MI355X-native 3-D U-Net training-step kernels and LMS swap engine (k3 library).

`paper_1811_12174_amd.k3` is the thin ctypes binding over the C-ABI declared in
include/k3.h; every operation runs in the HIP kernels of libk3.so.  There is no CPU
fallback: loading fails loudly when the library has not been built.
"""
from . import k3  # noqa: F401
