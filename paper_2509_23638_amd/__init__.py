"""MI355X-native MoE-layer hot path: thin Python binding over the C-ABI library.

Every step of the path runs in the HIP kernels of ``libmoe_hotpath.so``; this
package only marshals arguments (torch tensors -> raw device pointers).  There
is no CPU fallback: importing :mod:`paper_2509_23638_amd.binding` raises if the
library has not been built.
"""
from .build import build, LIB  # noqa: F401

__all__ = ["build", "LIB"]
