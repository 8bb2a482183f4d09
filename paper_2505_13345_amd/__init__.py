"""MI355X-native forward hot path of a collaboration-aware expert-parallel MoE layer.

csrc/      HIP kernels and the C ABI (include/occult.h), built into liboccult.so by build.py
binding.py ctypes marshalling, one function per C entry point
layer.py   device buffers and the call sequence of one layer
"""
from . import binding  # noqa: F401
from .binding import OccultError  # noqa: F401
