"""ctypes front end of the C oracle (direct_conv.c) -- TEST INFRASTRUCTURE ONLY.

Each function takes a shape object with the attributes N, Hin, Win, C, K, R, S,
SY, SX, DY, DX, PT, PL, PB, PR (the symbols of the paper's Listing 1) and numpy
arrays; the arithmetic itself is all in the C file.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liboracle.so")
_lib = None


class _Shape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("N", "Hin", "Win", "C", "K", "R", "S", "SY", "SX", "DY", "DX", "PT", "PL", "PB", "PR")]


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            from . import build as _b
            _b.build()
        lib = ctypes.CDLL(_LIB_PATH)
        lib.oracle_out_extent.restype = ctypes.c_int32
        lib.oracle_out_extent.argtypes = [ctypes.c_int32] * 6
        for fn in (lib.oracle_conv2d_f64, lib.oracle_conv2d_u8i8, lib.oracle_indirection,
                   lib.oracle_indirect_gemm_f64, lib.oracle_epilogue_f64, lib.oracle_epilogue_i32,
                   lib.oracle_requantise_u8):
            fn.restype = None
        _lib = lib
    return _lib


def _cshape(s) -> _Shape:
    return _Shape(*(int(getattr(s, f[0])) for f in _Shape._fields_))


def _ptr(a: np.ndarray):
    assert a.flags["C_CONTIGUOUS"]
    return ctypes.c_void_p(a.ctypes.data)


def num_threads() -> int:
    """Threads the OpenMP loops of the oracle will use."""
    env = os.environ.get("OMP_NUM_THREADS")
    if env:
        try:
            return max(1, int(env.split(",")[0]))
        except ValueError:
            pass
    return len(os.sched_getaffinity(0))


def set_num_threads(n: int) -> None:
    """Fix the number of OpenMP threads of the following calls (the paper's protocol is single-threaded)."""
    lib = _load()
    fn = lib.omp_set_num_threads          # from the OpenMP runtime the oracle is linked against
    fn.restype, fn.argtypes = None, [ctypes.c_int]
    fn(int(n))


def out_extent(s):
    """(Hout, Wout) by the floor formula stated in direct_conv.c."""
    lib = _load()
    return (lib.oracle_out_extent(s.Hin, s.PT, s.PB, s.DY, s.R, s.SY),
            lib.oracle_out_extent(s.Win, s.PL, s.PR, s.DX, s.S, s.SX))


def to_f64(a: np.ndarray) -> np.ndarray:
    """Exact widening to double.  uint16 arrays are bfloat16 bit patterns
    (a bfloat16 is the upper half of a float32)."""
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def _conv_f64(s, x, w, want_abs):
    lib = _load()
    x64 = np.ascontiguousarray(to_f64(x))
    w64 = np.ascontiguousarray(to_f64(w))
    assert x64.shape[:3] == (s.N, s.Hin, s.Win) and x64.shape[3] >= s.C
    assert w64.shape == (s.K, s.R, s.S, s.C)
    Hout, Wout = out_extent(s)
    out = np.zeros((s.N, Hout, Wout, s.K), dtype=np.float64)
    mag = np.zeros_like(out) if want_abs else None
    cs = _cshape(s)
    lib.oracle_conv2d_f64(ctypes.byref(cs), _ptr(x64), ctypes.c_int64(x64.shape[3]), _ptr(w64),
                          _ptr(out), _ptr(mag) if want_abs else None)
    return (out, mag) if want_abs else out


def conv2d(s, x, w) -> np.ndarray:
    """Direct convolution in double.  x: [N][Hin][Win][>=C], w: [K][R][S][C]
    (float32, float64 or bfloat16 bits as uint16).  Returns [N][Hout][Wout][K]."""
    return _conv_f64(s, x, w, False)


def conv2d_abs(s, x, w):
    """As conv2d, plus the per-output sum of |x*w| (scale of a rounding bound)."""
    return _conv_f64(s, x, w, True)


def conv2d_u8i8(s, x, w, zero_point: int, centred: bool = True) -> np.ndarray:
    """Quantised direct convolution, int32 accumulation (see direct_conv.c)."""
    lib = _load()
    assert x.dtype == np.uint8 and w.dtype == np.int8
    x = np.ascontiguousarray(x)
    w = np.ascontiguousarray(w)
    assert x.shape[:3] == (s.N, s.Hin, s.Win) and x.shape[3] >= s.C
    assert w.shape == (s.K, s.R, s.S, s.C)
    Hout, Wout = out_extent(s)
    out = np.zeros((s.N, Hout, Wout, s.K), dtype=np.int32)
    cs = _cshape(s)
    lib.oracle_conv2d_u8i8(ctypes.byref(cs), _ptr(x), ctypes.c_int64(x.shape[3]), _ptr(w),
                           ctypes.c_int32(zero_point), ctypes.c_int32(1 if centred else 0), _ptr(out))
    return out


def indirection(s) -> np.ndarray:
    """Logical indirection buffer: int32 [N*Hout*Wout][R*S], pixel index or -1."""
    lib = _load()
    Hout, Wout = out_extent(s)
    ent = np.empty((s.N * Hout * Wout, s.R * s.S), dtype=np.int32)
    cs = _cshape(s)
    lib.oracle_indirection(ctypes.byref(cs), _ptr(ent))
    return ent


def indirect_gemm(s, entries: np.ndarray, x, w) -> np.ndarray:
    """Listing-3-style evaluation through an indirection buffer, double accumulation."""
    lib = _load()
    x64 = np.ascontiguousarray(to_f64(x))
    w64 = np.ascontiguousarray(to_f64(w))
    entries = np.ascontiguousarray(entries, dtype=np.int32)
    Hout, Wout = out_extent(s)
    out = np.zeros((s.N, Hout, Wout, s.K), dtype=np.float64)
    zero = np.zeros(s.C, dtype=np.float64)
    cs = _cshape(s)
    lib.oracle_indirect_gemm_f64(ctypes.byref(cs), _ptr(entries), _ptr(x64), ctypes.c_int64(x64.shape[3]),
                                 _ptr(zero), _ptr(w64), _ptr(out))
    return out


def epilogue(y: np.ndarray, bias=None, relu: bool = False) -> np.ndarray:
    """Bias add and ReLU on the accumulators of conv2d / conv2d_u8i8 (float64 or int32, last axis = K)."""
    lib = _load()
    K = y.shape[-1]
    out = np.ascontiguousarray(y).copy()
    if out.dtype == np.int32:
        b = None if bias is None else np.ascontiguousarray(bias, dtype=np.int32)
        lib.oracle_epilogue_i32(_ptr(out), ctypes.c_int64(out.size), ctypes.c_int32(K),
                                _ptr(b) if b is not None else None, ctypes.c_int32(int(relu)))
    else:
        assert out.dtype == np.float64
        b = None if bias is None else np.ascontiguousarray(bias, dtype=np.float64)
        lib.oracle_epilogue_f64(_ptr(out), ctypes.c_int64(out.size), ctypes.c_int32(K),
                                _ptr(b) if b is not None else None, ctypes.c_int32(int(relu)))
    return out


def requantise_u8(y: np.ndarray, scale: float, out_zero_point: int) -> np.ndarray:
    """uint8 codes of an int32 result: clamp(rint(float32(y) * float32(scale)) + zero point, 0, 255)."""
    lib = _load()
    y = np.ascontiguousarray(y, dtype=np.int32)
    q = np.empty(y.shape, dtype=np.uint8)
    lib.oracle_requantise_u8(_ptr(y), ctypes.c_int64(y.size), ctypes.c_float(scale), ctypes.c_int32(out_zero_point),
                             _ptr(q))
    return q
