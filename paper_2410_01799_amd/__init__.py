"""MI355X-native signed cut decomposition (arXiv 2410.01799): C-ABI HIP library + thin binding.

``workloads`` (synthetic inputs, size arithmetic) imports without a GPU; ``scd`` is the ctypes
binding of ``libscd.so`` and raises if the library has not been built.
"""
from . import workloads  # noqa: F401

__all__ = ["workloads"]
