"""W4A16 mixed-precision matrix multiplication for MI355X (gfx950).

Y[M,N] (fp16) = X[M,K] (fp16) x s (W_int4[K,N] - z), fp32 accumulation
(Section 3, Eq. 2).  The arithmetic runs in the HIP library behind the C ABI
declared in include/w4a16.h; this package only marshals arguments.

Submodules are imported on demand so that the seeded input generators
(`workloads`) can be used where the HIP library is not built.
"""
import importlib

__all__ = ["binding", "workloads", "build"]


def __getattr__(name):
    if name in __all__:
        return importlib.import_module("." + name, __name__)
    raise AttributeError(name)
