"""Indirect Convolution (arXiv 1907.02129) for MI355X / gfx950.

The product is the C-ABI library libicv.so (HIP kernels, declared in
include/icv.h); `paper_1907_02129_amd.binding` is a thin ctypes layer over it
and `paper_1907_02129_amd.workloads` holds the seeded synthetic workloads.
Importing the package does not load the library; `load_library()` does, and
raises when it is missing.
"""
from .workloads import CONFIGS, HEADLINE, ConvShape, make_tensors  # noqa: F401


def load_library():
    import importlib
    return importlib.import_module(__name__ + ".binding").load_library()
