"""MI355X-native tile-centric mixed-precision GEMM (hand-written HIP behind a C ABI).

`gemm_mp` is the ctypes binding of libgemm_mp.so; `device` adds PyTorch plumbing (device
memory, streams) around it.  Nothing is loaded at import time.
"""
from . import gemm_mp  # noqa: F401

__all__ = ["gemm_mp"]
