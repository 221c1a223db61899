"""Deterministic, batch-invariant transformer decode step for AMD MI355X (gfx950).

A thin binding over libdetinfer's C ABI (include/detinfer.h): same names, same arguments, torch
tensors in place of raw pointers.  Every computation runs in the library's HIP kernels; torch is
used for device memory and streams only."""
from .api import *  # noqa: F401,F403
from .api import __all__  # noqa: F401
