"""CPU oracle for the ONNX contraction / pooling operators (test infrastructure only).

The arithmetic lives in ``onnx_oracle.c`` (plain C loop nests, double accumulation);
this module only compiles it with gcc, loads it with ctypes and marshals numpy
arrays.  Nothing here is used by the GPU library, and nothing here uses it.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "onnx_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None

_i64p = ctypes.POINTER(ctypes.c_int64)
_f32p = ctypes.POINTER(ctypes.c_float)
_f64p = ctypes.POINTER(ctypes.c_double)


def build(force=False):
    """Compile the oracle's C source into ``liboracle.so`` next to it."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_window_out.restype = ctypes.c_int64
        _lib.oracle_window_out.argtypes = [ctypes.c_int64] * 6 + [ctypes.c_int]
        ci, cf, c64 = ctypes.c_int, ctypes.c_float, ctypes.c_int64
        _lib.oracle_conv.argtypes = [_f32p, _i64p, _f32p, _i64p, _f32p, _i64p, _i64p, _i64p, c64,
                                     _f32p, ci, _f64p, _f64p]
        _lib.oracle_gemm.argtypes = [_f32p, _i64p, _f32p, _i64p, _f32p, _i64p, ci, cf, cf, ci, ci,
                                     ci, _f64p, _f64p]
        _lib.oracle_matmul.argtypes = [_f32p, _i64p, ci, _f32p, _i64p, ci, _f64p, _f64p, _i64p,
                                       ctypes.POINTER(ci)]
        _lib.oracle_maxpool.argtypes = [_f32p, _i64p, _i64p, _i64p, _i64p, _i64p, ci, _f32p, _i64p]
        _lib.oracle_avgpool.argtypes = [_f32p, _i64p, _i64p, _i64p, _i64p, ci, ci, _f64p]
        for f in (_lib.oracle_conv, _lib.oracle_gemm, _lib.oracle_matmul, _lib.oracle_maxpool,
                  _lib.oracle_avgpool):
            f.restype = ci
    return _lib


def _dims(v):
    v = [int(t) for t in v]
    return (ctypes.c_int64 * max(len(v), 1))(*v)


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(_f32p)


def _opt_f32(a):
    if a is None:
        return None, None
    return _f32(a)


def _check(rc, what):
    if rc != 0:
        raise ValueError("oracle %s rejected its arguments (code %d)" % (what, rc))


def window_out(n, k, pad_begin, pad_end, stride, dilation=1, ceil_mode=0):
    return int(_load().oracle_window_out(n, k, pad_begin, pad_end, stride, dilation, int(ceil_mode)))


def conv(X, W, B=None, pads=(0, 0, 0, 0), strides=(1, 1), dilations=(1, 1), group=1,
         residual=None, relu=False, want_scale=False):
    """ONNX Conv (+ optional residual add and Relu).  Returns float64 Y, or (Y, S)."""
    lib = _load()
    X, xp = _f32(X)
    W, wp = _f32(W)
    B, bp = _opt_f32(B)
    residual, rp = _opt_f32(residual)
    N, C, H, Wd = X.shape
    M, Cg, kH, kW = W.shape
    OH = window_out(H, kH, pads[0], pads[2], strides[0], dilations[0])
    OW = window_out(Wd, kW, pads[1], pads[3], strides[1], dilations[1])
    if OH < 0 or OW < 0:
        raise ValueError("oracle conv: window larger than padded input")
    if B is not None and B.shape != (M,):
        raise ValueError("oracle conv: bias shape")
    if residual is not None and residual.shape != (N, M, OH, OW):
        raise ValueError("oracle conv: residual shape")
    Y = np.empty((N, M, OH, OW), dtype=np.float64)
    S = np.empty_like(Y) if want_scale else None
    rc = lib.oracle_conv(xp, _dims(X.shape), wp, _dims(W.shape), bp, _dims(pads), _dims(strides),
                         _dims(dilations), int(group), rp, int(bool(relu)),
                         Y.ctypes.data_as(_f64p), S.ctypes.data_as(_f64p) if want_scale else None)
    _check(rc, "conv")
    return (Y, S) if want_scale else Y


def gemm(A, B, C=None, alpha=1.0, beta=1.0, transA=0, transB=0, relu=False, want_scale=False):
    """ONNX Gemm (+ optional Relu).  Returns float64 Y, or (Y, S)."""
    lib = _load()
    A, ap = _f32(A)
    B, bp = _f32(B)
    if A.ndim != 2 or B.ndim != 2:
        raise ValueError("oracle gemm: A and B must be 2-D")
    M = A.shape[1] if transA else A.shape[0]
    N = B.shape[0] if transB else B.shape[1]
    cp, cd, cr = None, _dims([]), 0
    if C is not None:
        C = np.ascontiguousarray(C, dtype=np.float32)
        cp, cd, cr = C.ctypes.data_as(_f32p), _dims(C.shape), C.ndim
    Y = np.empty((M, N), dtype=np.float64)
    S = np.empty_like(Y) if want_scale else None
    rc = lib.oracle_gemm(ap, _dims(A.shape), bp, _dims(B.shape), cp, cd, int(cr),
                         float(alpha), float(beta), int(transA),
                         int(transB), int(bool(relu)),
                         Y.ctypes.data_as(_f64p), S.ctypes.data_as(_f64p) if want_scale else None)
    _check(rc, "gemm")
    return (Y, S) if want_scale else Y


def matmul_shape(a_shape, b_shape):
    lib = _load()
    yd = (ctypes.c_int64 * 16)()
    yr = ctypes.c_int(0)
    rc = lib.oracle_matmul(None, _dims(a_shape), len(a_shape), None, _dims(b_shape), len(b_shape),
                           None, None, yd, ctypes.byref(yr))
    _check(rc, "matmul shape")
    return tuple(int(yd[i]) for i in range(yr.value))


def matmul(A, B, want_scale=False):
    """ONNX MatMul with numpy-style broadcasting.  Returns float64 Y, or (Y, S)."""
    lib = _load()
    A, ap = _f32(A)
    B, bp = _f32(B)
    shape = matmul_shape(A.shape, B.shape)
    Y = np.empty(shape, dtype=np.float64)
    S = np.empty_like(Y) if want_scale else None
    yd = (ctypes.c_int64 * 16)()
    yr = ctypes.c_int(0)
    rc = lib.oracle_matmul(ap, _dims(A.shape), A.ndim, bp, _dims(B.shape), B.ndim,
                           Y.ctypes.data_as(_f64p), S.ctypes.data_as(_f64p) if want_scale else None,
                           yd, ctypes.byref(yr))
    _check(rc, "matmul")
    return (Y, S) if want_scale else Y


def maxpool(X, kernel, pads=(0, 0, 0, 0), strides=(1, 1), dilations=(1, 1), ceil_mode=0,
            want_indices=True):
    """ONNX MaxPool.  Returns (Y float32, Indices int64) or Y."""
    lib = _load()
    X, xp = _f32(X)
    N, C, H, W = X.shape
    OH = window_out(H, kernel[0], pads[0], pads[2], strides[0], dilations[0], ceil_mode)
    OW = window_out(W, kernel[1], pads[1], pads[3], strides[1], dilations[1], ceil_mode)
    if OH < 0 or OW < 0:
        raise ValueError("oracle maxpool: window larger than padded input")
    Y = np.empty((N, C, OH, OW), dtype=np.float32)
    I = np.empty((N, C, OH, OW), dtype=np.int64) if want_indices else None
    rc = lib.oracle_maxpool(xp, _dims(X.shape), _dims(kernel), _dims(pads), _dims(strides),
                            _dims(dilations), int(ceil_mode), Y.ctypes.data_as(_f32p),
                            I.ctypes.data_as(_i64p) if want_indices else None)
    _check(rc, "maxpool")
    return (Y, I) if want_indices else Y


def avgpool(X, kernel=None, pads=(0, 0, 0, 0), strides=(1, 1), ceil_mode=0, count_include_pad=0):
    """ONNX AveragePool; ``kernel=None`` is GlobalAveragePool.  Returns float64 Y."""
    lib = _load()
    X, xp = _f32(X)
    N, C, H, W = X.shape
    if kernel is None:
        OH = OW = 1
        kp = pp = sp = None
    else:
        OH = window_out(H, kernel[0], pads[0], pads[2], strides[0], 1, ceil_mode)
        OW = window_out(W, kernel[1], pads[1], pads[3], strides[1], 1, ceil_mode)
        kp, pp, sp = _dims(kernel), _dims(pads), _dims(strides)
    if OH < 0 or OW < 0:
        raise ValueError("oracle avgpool: window larger than padded input")
    Y = np.empty((N, C, OH, OW), dtype=np.float64)
    rc = lib.oracle_avgpool(xp, _dims(X.shape), kp, pp, sp, int(ceil_mode),
                            int(count_include_pad), Y.ctypes.data_as(_f64p))
    _check(rc, "avgpool")
    return Y
