"""Indirect Convolution (arXiv 1907.02129) for MI355X / gfx950.

The product is the C-ABI library libicv.so (HIP kernels, declared in
include/icv.h); this package is a thin ctypes binding over it plus the seeded
workload generators.  Importing the package does not load the library;
`load_library()` does, and raises when it is missing.
"""
from .workloads import CONFIGS, HEADLINE, ConvShape, make_tensors  # noqa: F401


def load_library():
    from . import binding
    return binding.load_library()


def __getattr__(name):
    # binding symbols (icv_* wrappers, Conv2d helper) resolve lazily
    from . import binding
    try:
        return getattr(binding, name)
    except AttributeError as e:
        raise AttributeError(f"module {__name__!r} has no attribute {name!r}") from e
