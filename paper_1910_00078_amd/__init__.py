"""MI355X-native forward convolution with fused bias + activation (after arXiv 1910.00078).

The product is the C-ABI shared library libcvx.so (declared in include/cvx.h, built from csrc/ by
`python -m paper_1910_00078_amd.build`); `paper_1910_00078_amd.cvx` is its ctypes binding.
"""
from . import cvx  # noqa: F401

__all__ = ["cvx"]
