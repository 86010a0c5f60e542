"""ctypes binding of libicv.so: the same names as include/icv.h, argument marshalling only.

torch is used for device memory and streams; every step of the path runs in the
library's kernels.  There is no CPU fallback: when the library is missing or a
call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import numpy as np
import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libicv.so")

ICV_OK = 0
ICV_ERR_INVALID_ARG = -1
ICV_ERR_UNSUPPORTED = -2
ICV_ERR_HIP = -3
ICV_F32, ICV_BF16, ICV_U8I8 = 0, 1, 2
# icv_conv_params.plan: one algorithm, optionally or-ed with PLAN_PER_IMAGE (icv.h)
PLAN_VECTOR_ALU, PLAN_GATHER, PLAN_WINDOW, PLAN_FILTER_REGS = 1, 2, 3, 4
PLAN_PER_IMAGE = 8
DTYPES = {"f32": ICV_F32, "bf16": ICV_BF16, "u8i8": ICV_U8I8}

# every symbol include/icv.h declares
EXPORTS = (
    "icv_output_size", "icv_indirection_bytes", "icv_packed_filter_bytes", "icv_zero_row_bytes",
    "icv_im2col_bytes", "icv_indirection_index", "icv_get_indirection_layout", "icv_row_pixel_range",
    "icv_tile_span_bound", "icv_init_zero_row", "icv_pack_filter",
    "icv_setup_indirection", "icv_conv2d_nhwc", "icv_conv2d_nhwc_fused", "icv_im2col", "icv_gemm_nhwc", "icv_conv2d_nhwc_im2col",
    "icv_static_workspace_bytes", "icv_conv2d_nhwc_im2col_static",
    "icv_plan_name", "icv_status_string", "icv_last_hip_error", "icv_measure_mfma_peak",
)


class IcvError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = f"{where}: {status_string(status)} ({status})"
        if status == ICV_ERR_HIP:
            msg += f", hipError {_lib.icv_last_hip_error()}"
        super().__init__(msg)


class icv_conv_params(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "N", "Hin", "Win", "C", "K", "R", "S", "SY", "SX", "DY", "DX", "PT", "PL", "PB", "PR",
        "in_pixel_stride", "out_pixel_stride", "dtype", "input_zero_point", "plan")]


class icv_epilogue(ctypes.Structure):
    _fields_ = [("bias", ctypes.c_void_p), ("relu", ctypes.c_int32), ("out_type", ctypes.c_int32),
                ("out_scale", ctypes.c_float), ("out_zero_point", ctypes.c_int32)]


class icv_indirection_layout(ctypes.Structure):
    _fields_ = [("tile_rows", ctypes.c_int32), ("entry_bytes", ctypes.c_int32), ("zero_code", ctypes.c_int32),
                ("record_bytes", ctypes.c_int32), ("tiles", ctypes.c_int64), ("entries_at", ctypes.c_int64),
                ("records_at", ctypes.c_int64), ("int32_entries_at", ctypes.c_int64)]


ICV_OUT_ACC, ICV_OUT_BF16, ICV_OUT_U8 = 0, 1, 2

_lib = None


def load_library(path: str | None = None):
    """Load libicv.so (built in-tree by `python -m paper_1907_02129_amd.build`)."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    path = path or LIB_PATH
    if not os.path.exists(path):
        raise RuntimeError(f"{path} not found: build it with `python -m paper_1907_02129_amd.build`")
    lib = ctypes.CDLL(path)
    P = ctypes.POINTER(icv_conv_params)
    vp, i32p = ctypes.c_void_p, ctypes.POINTER(ctypes.c_int32)
    sig = {
        "icv_output_size": (ctypes.c_int, [P, i32p, i32p]),
        "icv_indirection_bytes": (ctypes.c_size_t, [P]),
        "icv_packed_filter_bytes": (ctypes.c_size_t, [P]),
        "icv_zero_row_bytes": (ctypes.c_size_t, [P]),
        "icv_im2col_bytes": (ctypes.c_size_t, [P]),
        "icv_indirection_index": (ctypes.c_int64, [P, ctypes.c_int64, ctypes.c_int32]),
        "icv_get_indirection_layout": (ctypes.c_int, [P, ctypes.POINTER(icv_indirection_layout)]),
        "icv_row_pixel_range": (ctypes.c_int, [P, ctypes.c_int64, ctypes.c_int64, ctypes.POINTER(ctypes.c_int64),
                                               ctypes.POINTER(ctypes.c_int64)]),
        "icv_tile_span_bound": (ctypes.c_int64, [P, ctypes.c_int32]),
        "icv_init_zero_row": (ctypes.c_int, [P, vp, vp]),
        "icv_pack_filter": (ctypes.c_int, [P, vp, vp, vp]),
        "icv_setup_indirection": (ctypes.c_int, [P, vp, vp]),
        "icv_conv2d_nhwc": (ctypes.c_int, [P, vp, vp, vp, vp, vp, vp]),
        "icv_conv2d_nhwc_fused": (ctypes.c_int, [P, vp, vp, vp, vp, ctypes.POINTER(icv_epilogue), vp, vp]),
        "icv_im2col": (ctypes.c_int, [P, vp, vp, vp]),
        "icv_gemm_nhwc": (ctypes.c_int, [P, vp, vp, vp, vp]),
        "icv_conv2d_nhwc_im2col": (ctypes.c_int, [P, vp, vp, vp, vp, vp]),
        "icv_static_workspace_bytes": (ctypes.c_size_t, []),
        "icv_conv2d_nhwc_im2col_static": (ctypes.c_int, [P, vp, vp, vp, vp]),
        "icv_plan_name": (ctypes.c_char_p, [P]),
        "icv_measure_mfma_peak": (ctypes.c_int, [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.POINTER(ctypes.c_double),
                                                 ctypes.c_void_p]),
        "icv_status_string": (ctypes.c_char_p, [ctypes.c_int]),
        "icv_last_hip_error": (ctypes.c_int, []),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    _lib = lib
    return lib


def make_params(shape, plan: int = 0, in_pixel_stride: int = 0, out_pixel_stride: int = 0) -> icv_conv_params:
    """icv_conv_params from a workloads.ConvShape-like object."""
    return icv_conv_params(
        shape.N, shape.Hin, shape.Win, shape.C, shape.K, shape.R, shape.S, shape.SY, shape.SX, shape.DY,
        shape.DX, shape.PT, shape.PL, shape.PB, shape.PR, in_pixel_stride, out_pixel_stride,
        DTYPES[shape.dtype], getattr(shape, "zero_point", 0), plan)


def _check(status: int, where: str):
    if status != ICV_OK:
        raise IcvError(status, where)


def _ptr(t) -> ctypes.c_void_p:
    if t is None:
        return ctypes.c_void_p(0)
    if isinstance(t, int):
        return ctypes.c_void_p(t)
    if not t.is_cuda:
        raise ValueError("icv takes device tensors")
    if not t.is_contiguous():
        raise ValueError("icv takes contiguous tensors")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream=None) -> ctypes.c_void_p:
    s = stream if stream is not None else torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


# ---------------------------------------------------------------- thin wrappers, same names as the header
def status_string(status: int) -> str:
    return load_library().icv_status_string(status).decode()


def measure_mfma_peak(dtype: str, waves_per_simd: int = 2, varied_operands: bool = False) -> float:
    """Operations per second of a register-only tensor-core loop on the current device (icv_measure_mfma_peak)."""
    v = ctypes.c_double(0.0)
    _check(load_library().icv_measure_mfma_peak(DTYPES[dtype], waves_per_simd, int(varied_operands), ctypes.byref(v), _stream()),
           "icv_measure_mfma_peak")
    return v.value


def plan_name(p: icv_conv_params) -> str:
    return load_library().icv_plan_name(ctypes.byref(p)).decode()


def output_size(p: icv_conv_params):
    h, w = ctypes.c_int32(), ctypes.c_int32()
    _check(load_library().icv_output_size(ctypes.byref(p), ctypes.byref(h), ctypes.byref(w)), "icv_output_size")
    return h.value, w.value


def indirection_bytes(p) -> int:
    return load_library().icv_indirection_bytes(ctypes.byref(p))


def packed_filter_bytes(p) -> int:
    return load_library().icv_packed_filter_bytes(ctypes.byref(p))


def zero_row_bytes(p) -> int:
    return load_library().icv_zero_row_bytes(ctypes.byref(p))


def im2col_bytes(p) -> int:
    return load_library().icv_im2col_bytes(ctypes.byref(p))


def indirection_index(p, m: int, tap: int) -> int:
    return load_library().icv_indirection_index(ctypes.byref(p), m, tap)


def get_indirection_layout(p) -> icv_indirection_layout:
    L = icv_indirection_layout()
    _check(load_library().icv_get_indirection_layout(ctypes.byref(p), ctypes.byref(L)), "icv_get_indirection_layout")
    return L


def row_pixel_range(p, m0: int, m1: int):
    a, b = ctypes.c_int64(), ctypes.c_int64()
    _check(load_library().icv_row_pixel_range(ctypes.byref(p), m0, m1, ctypes.byref(a), ctypes.byref(b)),
           "icv_row_pixel_range")
    return a.value, b.value


def tile_span_bound(p, rows: int) -> int:
    return load_library().icv_tile_span_bound(ctypes.byref(p), rows)


def init_zero_row(p, zero_row, stream=None):
    _check(load_library().icv_init_zero_row(ctypes.byref(p), _ptr(zero_row), _stream(stream)), "icv_init_zero_row")


def pack_filter(p, filter_krsc, packed, stream=None):
    _check(load_library().icv_pack_filter(ctypes.byref(p), _ptr(filter_krsc), _ptr(packed), _stream(stream)),
           "icv_pack_filter")


def setup_indirection(p, indirection, stream=None):
    _check(load_library().icv_setup_indirection(ctypes.byref(p), _ptr(indirection), _stream(stream)),
           "icv_setup_indirection")


def conv2d_nhwc(p, input, packed_filter, indirection, zero_row, output, stream=None):
    _check(load_library().icv_conv2d_nhwc(ctypes.byref(p), _ptr(input), _ptr(packed_filter), _ptr(indirection),
                                          _ptr(zero_row), _ptr(output), _stream(stream)), "icv_conv2d_nhwc")


def conv2d_nhwc_fused(p, input, packed_filter, indirection, zero_row, epilogue, output, stream=None):
    _check(load_library().icv_conv2d_nhwc_fused(ctypes.byref(p), _ptr(input), _ptr(packed_filter), _ptr(indirection),
                                                _ptr(zero_row), ctypes.byref(epilogue), _ptr(output),
                                                _stream(stream)), "icv_conv2d_nhwc_fused")


def make_epilogue(bias=None, relu=False, out_type=ICV_OUT_ACC, out_scale=1.0, out_zero_point=0) -> icv_epilogue:
    """icv_epilogue; `bias` is a device tensor (float32, or int32 for u8i8) that the caller keeps alive."""
    return icv_epilogue(bias.data_ptr() if bias is not None else None, int(relu), out_type, out_scale,
                        out_zero_point)


def im2col(p, input, ws, stream=None):
    _check(load_library().icv_im2col(ctypes.byref(p), _ptr(input), _ptr(ws), _stream(stream)), "icv_im2col")


def gemm_nhwc(p, ws, packed_filter, output, stream=None):
    _check(load_library().icv_gemm_nhwc(ctypes.byref(p), _ptr(ws), _ptr(packed_filter), _ptr(output),
                                        _stream(stream)), "icv_gemm_nhwc")


def conv2d_nhwc_im2col(p, input, packed_filter, ws, output, stream=None):
    _check(load_library().icv_conv2d_nhwc_im2col(ctypes.byref(p), _ptr(input), _ptr(packed_filter), _ptr(ws),
                                                 _ptr(output), _stream(stream)), "icv_conv2d_nhwc_im2col")


def static_workspace_bytes() -> int:
    return load_library().icv_static_workspace_bytes()


def conv2d_nhwc_im2col_static(p, input, packed_filter, output, stream=None):
    _check(load_library().icv_conv2d_nhwc_im2col_static(ctypes.byref(p), _ptr(input), _ptr(packed_filter), _ptr(output),
                                                        _stream(stream)), "icv_conv2d_nhwc_im2col_static")


# ---------------------------------------------------------------- convenience: buffers for one problem
def to_device(a: np.ndarray, device="cuda:0") -> torch.Tensor:
    """numpy -> device tensor; uint16 arrays are bfloat16 bit patterns."""
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(a).to(device)


@dataclass
class ConvBuffers:
    """Device buffers of one convolution problem (allocated through torch, filled by the library)."""
    p: icv_conv_params
    Hout: int
    Wout: int
    zero_row: torch.Tensor
    packed: torch.Tensor
    indirection: torch.Tensor
    output: torch.Tensor

    @property
    def M(self) -> int:
        return self.p.N * self.Hout * self.Wout


def prepare(shape, filter_dev: torch.Tensor, plan: int = 0, device="cuda:0", in_pixel_stride: int = 0,
            out_pixel_stride: int = 0) -> ConvBuffers:
    """Set-up phase: zero row, packed filter, indirection buffer, output tensor."""
    p = make_params(shape, plan, in_pixel_stride, out_pixel_stride)
    Hout, Wout = output_size(p)
    zero_row = torch.empty(zero_row_bytes(p), dtype=torch.uint8, device=device)
    packed = torch.empty(packed_filter_bytes(p), dtype=torch.uint8, device=device)
    ind = torch.empty(indirection_bytes(p) // 4, dtype=torch.int32, device=device)
    out_dtype = torch.int32 if shape.dtype == "u8i8" else torch.float32
    ostride = out_pixel_stride or shape.K
    out = torch.empty((shape.N, Hout, Wout, ostride), dtype=out_dtype, device=device)
    init_zero_row(p, zero_row)
    pack_filter(p, filter_dev, packed)
    setup_indirection(p, ind)
    return ConvBuffers(p, Hout, Wout, zero_row, packed, ind, out)


def run(buf: ConvBuffers, input_dev: torch.Tensor) -> torch.Tensor:
    conv2d_nhwc(buf.p, input_dev, buf.packed, buf.indirection, buf.zero_row, buf.output)
    return buf.output


def stored_for_tensor_cores(shape):
    """The shape as its tensors would be kept in memory for the tensor-core kernels.  16-bit / 8-bit tensors: 3
    channels are stored as 4 (an 8-byte pixel); counts that are neither 4, 8, 16 nor a multiple of 32 are rounded up
    to a multiple of 32 (64-byte rows).  fp32 tensors: counts are rounded up to a multiple of 16 (64-byte rows).  The
    padding channels of input and filter hold zeros and `c_logical` keeps the real count (FLOPs are counted on it).
    Shapes that need no padding are returned as they are; the unpadded shape is always valid too and runs on the
    vector-ALU kernel."""
    C = shape.C
    if shape.dtype == "f32":
        Cs = -(-C // 16) * 16
    elif C == 3:
        Cs = 4
    elif C % 32 == 0 or C in (4, 8, 16):
        Cs = C
    else:
        Cs = -(-C // 32) * 32
    if Cs == C:
        return shape
    return shape.with_(C=Cs, c_logical=C)
