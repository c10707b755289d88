"""MI355X-native convolution library (Winograd F(n,k) / 1x1 GEMM / direct + planner).

Thin ctypes binding over libmnnconv.so; every step of the path runs in the HIP
kernels behind the C ABI declared in include/mnn_conv.h.  The binding is loaded
on first use so that ``paper_2002_12418_amd.build`` can be imported (and the
library rebuilt) without loading a stale shared object.
"""
import importlib

_binding = None


def __getattr__(name):
    global _binding
    if name.startswith("__"):
        raise AttributeError(name)
    if _binding is None:
        _binding = importlib.import_module(".binding", __name__)
    try:
        return getattr(_binding, name)
    except AttributeError:
        raise AttributeError(f"module {__name__!r} has no attribute {name!r}") from None
