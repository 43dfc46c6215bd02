"""nz: MI355X-native per-rank compression path (quantize -> select -> encode, decode, fused reduce).

The compute lives in the HIP library csrc/ -> libnz.so behind the C ABI of
include/nz.h; `binding` marshals arguments for it.  Importing this package
loads nothing; the binding loads the library on first use and raises if it is
missing (there is no CPU fallback).
"""
__all__ = ["binding", "workloads"]
