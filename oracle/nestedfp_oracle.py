"""ctypes/numpy front end of the C oracle (test infrastructure only).

Arrays in, arrays out; no arithmetic of the method lives here -- every value is
produced by ``nestedfp_oracle.c``.  FP16 tensors travel as ``uint16`` bit
patterns (``numpy.float16`` arrays are viewed, never converted).
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "nestedfp_oracle.c")
_LIB = os.path.join(_HERE, "libnestedfp_oracle.so")
_lib = None


def build_oracle(force=False):
    """Compile the C oracle with gcc (a second or two)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-std=c11", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build_oracle()
    lib = ctypes.CDLL(_LIB)
    c = ctypes
    u8p, u16p, f32p, f64p = (c.POINTER(c.c_uint8), c.POINTER(c.c_uint16),
                             c.POINTER(c.c_float), c.POINTER(c.c_double))
    i64 = c.c_int64
    lib.oracle_fp16_value.restype = c.c_double
    lib.oracle_fp16_value.argtypes = [c.c_uint16]
    lib.oracle_e4m3_value.restype = c.c_double
    lib.oracle_e4m3_value.argtypes = [c.c_uint8]
    lib.oracle_e4m3_encode.restype = c.c_uint8
    lib.oracle_e4m3_encode.argtypes = [c.c_double]
    lib.oracle_in_range.restype = c.c_int
    lib.oracle_in_range.argtypes = [c.c_uint16]
    lib.oracle_decompose_one.restype = None
    lib.oracle_decompose_one.argtypes = [c.c_uint16, u8p, u8p]
    lib.oracle_reconstruct_one.restype = c.c_uint16
    lib.oracle_reconstruct_one.argtypes = [c.c_uint8, c.c_uint8]
    lib.oracle_decompose.restype = c.c_uint64
    lib.oracle_decompose.argtypes = [u16p, i64, i64, i64, u8p, u8p]
    lib.oracle_count_out_of_range.restype = c.c_uint64
    lib.oracle_count_out_of_range.argtypes = [u16p, i64, i64, i64]
    lib.oracle_reconstruct.restype = None
    lib.oracle_reconstruct.argtypes = [u8p, u8p, i64, i64, u16p, i64]
    lib.oracle_quantize_act.restype = None
    lib.oracle_quantize_act.argtypes = [u16p, i64, i64, i64, f32p, u8p, f32p]
    lib.oracle_gemm_fp16.restype = None
    lib.oracle_gemm_fp16.argtypes = [u16p, i64, i64, i64, u16p, i64, i64, f64p, i64]
    lib.oracle_gemm_fp16_planes.restype = None
    lib.oracle_gemm_fp16_planes.argtypes = [u16p, i64, i64, i64, u8p, u8p, i64, f64p, i64]
    lib.oracle_gemm_fp8.restype = None
    lib.oracle_gemm_fp8.argtypes = [u8p, f32p, i64, i64, u8p, i64, f64p, i64]
    lib.oracle_dot_fp16.restype = c.c_double
    lib.oracle_dot_fp16.argtypes = [u16p, u16p, i64]
    lib.oracle_dot_fp8.restype = c.c_double
    lib.oracle_dot_fp8.argtypes = [u8p, c.c_float, u8p, i64]
    _lib = lib
    return lib


def _bits(a):
    """2-D contiguous uint16 view of an fp16 / uint16 array."""
    a = np.asarray(a)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    if a.dtype != np.uint16:
        raise TypeError("expected float16 or uint16, got %s" % a.dtype)
    return np.ascontiguousarray(a)


def _u8(a):
    a = np.asarray(a)
    if a.dtype != np.uint8:
        raise TypeError("expected uint8, got %s" % a.dtype)
    return np.ascontiguousarray(a)


def _p(a, ty):
    return a.ctypes.data_as(ctypes.POINTER(ty))


# ---- scalars ----------------------------------------------------------------

def fp16_value(bits):
    return _load().oracle_fp16_value(int(bits))


def e4m3_value(code):
    return _load().oracle_e4m3_value(int(code))


def e4m3_encode(v):
    return _load().oracle_e4m3_encode(float(v))


def in_range(bits):
    return bool(_load().oracle_in_range(int(bits)))


def decompose_one(bits):
    up, lo = ctypes.c_uint8(), ctypes.c_uint8()
    _load().oracle_decompose_one(int(bits), ctypes.byref(up), ctypes.byref(lo))
    return up.value, lo.value


def reconstruct_one(upper, lower):
    return _load().oracle_reconstruct_one(int(upper), int(lower))


# ---- tensors ----------------------------------------------------------------

def decompose(W):
    """W: [N,K] fp16/uint16 -> (upper u8 [N,K], lower u8 [N,K], n_out_of_range)."""
    Wb = _bits(W)
    N, K = Wb.shape
    upper = np.empty((N, K), np.uint8)
    lower = np.empty((N, K), np.uint8)
    bad = _load().oracle_decompose(_p(Wb, ctypes.c_uint16), N, K, K,
                                   _p(upper, ctypes.c_uint8), _p(lower, ctypes.c_uint8))
    return upper, lower, int(bad)


def count_out_of_range(W):
    Wb = _bits(W)
    N, K = Wb.shape
    return int(_load().oracle_count_out_of_range(_p(Wb, ctypes.c_uint16), N, K, K))


def reconstruct(upper, lower):
    """planes [N,K] u8 -> W bits uint16 [N,K]."""
    up, lo = _u8(upper), _u8(lower)
    N, K = up.shape
    W = np.empty((N, K), np.uint16)
    _load().oracle_reconstruct(_p(up, ctypes.c_uint8), _p(lo, ctypes.c_uint8), N, K,
                               _p(W, ctypes.c_uint16), K)
    return W


def quantize_act(X, static_scale=None):
    """X [M,K] fp16 -> (Xq u8 [M,K], scales f32 [M])."""
    Xb = _bits(X)
    M, K = Xb.shape
    Xq = np.empty((M, K), np.uint8)
    scales = np.empty((M,), np.float32)
    ss = None
    if static_scale is not None:
        ss = ctypes.byref(ctypes.c_float(float(static_scale)))
    _load().oracle_quantize_act(_p(Xb, ctypes.c_uint16), M, K, K, ss,
                                _p(Xq, ctypes.c_uint8), _p(scales, ctypes.c_float))
    return Xq, scales


def gemm_fp16(X, W):
    """Y[m,n] = sum_k X[m,k] W[n,k] in fp64; X [M,K], W [N,K] fp16."""
    Xb, Wb = _bits(X), _bits(W)
    M, K = Xb.shape
    N, K2 = Wb.shape
    assert K == K2
    Y = np.empty((M, N), np.float64)
    _load().oracle_gemm_fp16(_p(Xb, ctypes.c_uint16), M, K, K, _p(Wb, ctypes.c_uint16), N, K,
                             _p(Y, ctypes.c_double), N)
    return Y


def gemm_fp16_planes(X, upper, lower):
    Xb, up, lo = _bits(X), _u8(upper), _u8(lower)
    M, K = Xb.shape
    N, K2 = up.shape
    assert K == K2 and lo.shape == up.shape
    Y = np.empty((M, N), np.float64)
    _load().oracle_gemm_fp16_planes(_p(Xb, ctypes.c_uint16), M, K, K, _p(up, ctypes.c_uint8),
                                    _p(lo, ctypes.c_uint8), N, _p(Y, ctypes.c_double), N)
    return Y


def gemm_fp8(Xq, scales, upper):
    """FP8 mode from already-quantised activations; never takes the lower plane."""
    xq, up = _u8(Xq), _u8(upper)
    sc = np.ascontiguousarray(np.asarray(scales, np.float32))
    M, K = xq.shape
    N, K2 = up.shape
    assert K == K2 and sc.shape == (M,)
    Y = np.empty((M, N), np.float64)
    _load().oracle_gemm_fp8(_p(xq, ctypes.c_uint8), _p(sc, ctypes.c_float), M, K,
                            _p(up, ctypes.c_uint8), N, _p(Y, ctypes.c_double), N)
    return Y


def dot_fp16(x_row, w_row):
    xb, wb = _bits(x_row).reshape(-1), _bits(w_row).reshape(-1)
    assert xb.shape == wb.shape
    return _load().oracle_dot_fp16(_p(xb, ctypes.c_uint16), _p(wb, ctypes.c_uint16), xb.size)


def dot_fp8(xq_row, scale, upper_row):
    xq, up = _u8(xq_row).reshape(-1), _u8(upper_row).reshape(-1)
    assert xq.shape == up.shape
    return _load().oracle_dot_fp8(_p(xq, ctypes.c_uint8), float(scale), _p(up, ctypes.c_uint8),
                                  xq.size)
