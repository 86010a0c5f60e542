"""CPU oracle -- TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package.  It shares no code with the HIP library and never imports it.
"""
from .direct_conv import (  # noqa: F401
    out_extent, conv2d, conv2d_abs, conv2d_u8i8, indirection, indirect_gemm, to_f64, num_threads, epilogue,
    requantise_u8, set_num_threads,
)
