"""MI355X (gfx950) library for the hot path of encoding-decomposition quantized networks.

`paper_1905_13389_amd.qnn` is a thin ctypes binding over the C ABI declared in include/qnn.h
(argument marshalling only; every step runs in the HIP kernels of libqnn.so).
"""
from . import qnn  # noqa: F401
