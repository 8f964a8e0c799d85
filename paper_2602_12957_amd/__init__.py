"""MI355X-native verification hot path of Hierarchical Speculative Decoding.

The product is the C-ABI shared library `libhsd.so` (sources in csrc/, declarations in include/hsd.h).
`binding` mirrors its entry points one to one through ctypes; `runtime.Engine` only allocates device
buffers through torch and marshals arguments.  There is no CPU or PyTorch fallback: if the library has
not been built, importing `binding` raises.
"""
from . import build as _build  # noqa: F401

__all__ = ["binding", "runtime", "build"]
