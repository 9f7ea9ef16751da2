"""ctypes binding of libonnxhip.so: same names and argument order as include/onnxhip.h.

Argument marshalling only.  Tensors are torch CUDA tensors (fp32, contiguous); torch supplies
device memory and the current stream, every operator's arithmetic runs in the library.
Each compute wrapper allocates the result with torch.empty unless ``out=`` is given.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libonnxhip.so")

ONNX_OK = 0
ONNX_ERR_UNSUPPORTED = 5
ACT_NONE, ACT_RELU = 0, 1
STATUS_NAMES = {1: "ONNX_ERR_NULL", 2: "ONNX_ERR_RANK", 3: "ONNX_ERR_SHAPE", 4: "ONNX_ERR_ATTR",
                5: "ONNX_ERR_UNSUPPORTED", 6: "ONNX_ERR_ALIAS", 7: "ONNX_ERR_DEVICE"}


class OnnxHipError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("%s: %s" % (STATUS_NAMES.get(status, status), message))
        self.status = status


def lib_path():
    return _LIB_PATH


if not os.path.exists(_LIB_PATH):
    raise ImportError("libonnxhip.so is not built (%s); run `python -m paper_2008_08272_amd.build` "
                      "or __graft_entry__.build() first -- there is no fallback path" % _LIB_PATH)

_lib = ctypes.CDLL(_LIB_PATH)
_i64p = ctypes.POINTER(ctypes.c_int64)
_vp, _ci, _cf, _c64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_int64
_lib.onnx_last_error.restype = ctypes.c_char_p
_lib.onnx_conv_infer.argtypes = [_i64p, _i64p, _i64p, _i64p, _i64p, _c64, _i64p]
_lib.onnx_pool_infer.argtypes = [_i64p, _i64p, _i64p, _i64p, _i64p, _ci, _i64p]
_lib.onnx_matmul_infer.argtypes = [_i64p, _ci, _i64p, _ci, _i64p, ctypes.POINTER(_ci)]
_lib.onnx_conv.argtypes = [_vp, _i64p, _vp, _i64p, _vp, _i64p, _i64p, _i64p, _c64, _vp, _ci, _vp, _i64p, _vp]
_lib.onnx_conv_fixed_scratch.argtypes = _lib.onnx_conv.argtypes
_lib.onnx_conv_fixed_scratch.restype = _ci
_lib.onnx_last_launch.restype = ctypes.c_char_p
CONV_FIXED_SCRATCH_BYTES = 16 << 20
CONV_FIXED_SCRATCH_MAX_OUTPUTS = 1 << 21
_lib.onnx_gemm.argtypes = [_vp, _i64p, _vp, _i64p, _vp, _i64p, _ci, _cf, _cf, _ci, _ci, _ci, _vp, _i64p, _vp]
_lib.onnx_matmul.argtypes = [_vp, _i64p, _ci, _vp, _i64p, _ci, _vp, _i64p, _ci, _vp]
_lib.onnx_maxpool.argtypes = [_vp, _i64p, _i64p, _i64p, _i64p, _i64p, _ci, _vp, _vp, _i64p, _vp]
_lib.onnx_avgpool.argtypes = [_vp, _i64p, _i64p, _i64p, _i64p, _ci, _ci, _vp, _i64p, _vp]
_lib.onnx_maxpool_lp.argtypes = [_vp, _i64p, _i64p, _i64p, _i64p, _i64p, _ci, _vp, _i64p, _ci, _vp]
_lib.onnx_avgpool_lp.argtypes = [_vp, _i64p, _i64p, _i64p, _i64p, _ci, _ci, _vp, _i64p, _ci, _vp]
_lib.onnx_leakyrelu_lp.argtypes = [_vp, _c64, _cf, _vp, _ci, _vp]
_lib.onnx_leakyrelu_lp.restype = _ci
_lib.onnx_add_lp.argtypes = [_vp, _i64p, _ci, _vp, _i64p, _ci, _vp, _i64p, _ci, _ci, _vp]
_lib.onnx_add_lp.restype = _ci
_lib.onnx_abs_lp.argtypes = [_vp, _c64, _vp, _ci, _vp]
_lib.onnx_abs_lp.restype = _ci
_lib.onnx_reducesum_lp.argtypes = [_vp, _i64p, _ci, _i64p, _ci, _ci, _vp, _i64p, _ci, _ci, _vp]
_lib.onnx_reducesum_lp.restype = _ci
_lib.onnx_softmax_lp.argtypes = [_vp, _i64p, _ci, _ci, _vp, _ci, _vp]
_lib.onnx_softmax_lp.restype = _ci
for _f in (_lib.onnx_conv_infer, _lib.onnx_pool_infer, _lib.onnx_matmul_infer, _lib.onnx_conv,
           _lib.onnx_gemm, _lib.onnx_matmul, _lib.onnx_maxpool, _lib.onnx_avgpool, _lib.onnx_maxpool_lp,
           _lib.onnx_avgpool_lp):
    _f.restype = _ci

_ip = ctypes.POINTER(_ci)
_lib.onnx_broadcast_infer.argtypes = [_i64p, _ci, _i64p, _ci, _i64p, _ip]
_lib.onnx_reduce_infer.argtypes = [_i64p, _ci, _i64p, _ci, _ci, _i64p, _ip]
_lib.onnx_add.argtypes = [_vp, _i64p, _ci, _vp, _i64p, _ci, _vp, _i64p, _ci, _vp]
_lib.onnx_relu.argtypes = [_vp, _c64, _vp, _vp]
_lib.onnx_leakyrelu.argtypes = [_vp, _c64, _cf, _vp, _vp]
_lib.onnx_abs.argtypes = [_vp, _c64, _vp, _vp]
_lib.onnx_reducesum.argtypes = [_vp, _i64p, _ci, _i64p, _ci, _ci, _vp, _i64p, _ci, _vp]
_lib.onnx_softmax.argtypes = [_vp, _i64p, _ci, _ci, _vp, _vp]
for _f in (_lib.onnx_broadcast_infer, _lib.onnx_reduce_infer, _lib.onnx_add, _lib.onnx_relu, _lib.onnx_leakyrelu,
           _lib.onnx_abs, _lib.onnx_reducesum, _lib.onnx_softmax):
    _f.restype = _ci
_lib.onnx_gemm_lp.argtypes = [_vp, _i64p, _vp, _i64p, _vp, _i64p, _ci, _cf, _cf, _ci, _ci, _ci, _vp, _i64p, _ci, _ci, _vp]
_lib.onnx_gemm_lp.restype = _ci
F32, F16, BF16 = 0, 1, 2
_lib.onnx_matmul_lp.argtypes = [_vp, _i64p, _ci, _vp, _i64p, _ci, _vp, _i64p, _ci, _ci, _ci, _vp]
_lib.onnx_matmul_lp.restype = _ci
_lib.onnx_conv_lp.argtypes = [_vp, _i64p, _vp, _i64p, _vp, _i64p, _i64p, _i64p, _c64, _vp, _ci, _vp, _i64p, _ci, _ci, _vp]
_lib.onnx_conv_lp.restype = _ci
_lib.onnx_conv_lp_taps.argtypes = _lib.onnx_conv_lp.argtypes
_lib.onnx_conv_lp_taps.restype = _ci
_lib.onnx_conv_lp_filter_taps.argtypes = [_vp, _i64p, _vp, _vp]
_lib.onnx_conv_lp_filter_taps.restype = _ci
_lib.onnx_lstm_scratch_bytes.argtypes = [_i64p, _c64, _ci]
_lib.onnx_lstm_scratch_bytes.restype = ctypes.c_size_t
_lib.onnx_lstm.argtypes = [_vp, _i64p, _vp, _vp, _vp, _vp, _vp, _c64, _ci, _vp, _vp, _vp, _vp, ctypes.c_size_t, _vp]
_lib.onnx_lstm.restype = _ci
LSTM_DIRECTIONS = {"forward": 0, "reverse": 1, "bidirectional": 2}



class ChainOp(ctypes.Structure):
    """onnx_chain_op of include/onnxhip.h."""
    _fields_ = [("kind", ctypes.c_int32), ("act", ctypes.c_int32), ("outputs", ctypes.c_int64),
                ("kernel", ctypes.c_int64 * 2), ("pads", ctypes.c_int64 * 4), ("strides", ctypes.c_int64 * 2),
                ("dilations", ctypes.c_int64 * 2), ("ceil_mode", ctypes.c_int32),
                ("count_include_pad", ctypes.c_int32), ("transB", ctypes.c_int32), ("alpha", ctypes.c_float),
                ("beta", ctypes.c_float), ("W", ctypes.c_void_p), ("B", ctypes.c_void_p), ("Y", ctypes.c_void_p)]


_lib.onnx_chain.argtypes = [ctypes.POINTER(ChainOp), _ci, _vp, _i64p, _vp]
_lib.onnx_chain.restype = _ci
_lib.onnx_set_workspace.argtypes = [_vp, ctypes.c_size_t]
_lib.onnx_set_workspace.restype = _ci
_workspace_tensor = None


def onnx_set_workspace(tensor):
    """Hand a uint8 / float32 CUDA tensor to the library as split-K scratch (None removes it).
    The binding keeps a reference so the memory outlives the calls that use it."""
    global _workspace_tensor
    if tensor is None:
        _check(_lib.onnx_set_workspace(None, 0))
        _workspace_tensor = None
        return
    if not (tensor.is_cuda and tensor.is_contiguous()):
        raise TypeError("the workspace must be a contiguous tensor on the GPU")
    _check(_lib.onnx_set_workspace(ctypes.c_void_p(tensor.data_ptr()), tensor.numel() * tensor.element_size()))
    _workspace_tensor = tensor


def onnx_last_error():
    return _lib.onnx_last_error().decode()


def onnx_last_launch():
    return _lib.onnx_last_launch().decode()


def _check(st):
    if st != ONNX_OK:
        raise OnnxHipError(st, onnx_last_error())


def dims(v):
    v = [int(t) for t in v]
    return (ctypes.c_int64 * max(len(v), 1))(*v)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _dev(t, name):
    if t is None:
        return None
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()):
        raise TypeError("%s must be a contiguous float32 tensor on the GPU" % name)
    return t


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def raw():
    """The loaded ctypes library (for callers that prebuild their argument lists)."""
    return _lib


def onnx_conv_infer(x_dims, w_dims, pads=(0, 0, 0, 0), strides=(1, 1), dilations=(1, 1), group=1):
    y = (ctypes.c_int64 * 4)()
    _check(_lib.onnx_conv_infer(dims(x_dims), dims(w_dims), dims(pads), dims(strides), dims(dilations),
                                int(group), y))
    return tuple(y)


def onnx_pool_infer(x_dims, kernel, pads=(0, 0, 0, 0), strides=(1, 1), dilations=(1, 1), ceil_mode=0):
    y = (ctypes.c_int64 * 4)()
    _check(_lib.onnx_pool_infer(dims(x_dims), dims(kernel), dims(pads), dims(strides), dims(dilations),
                                int(ceil_mode), y))
    return tuple(y)


def onnx_matmul_infer(a_dims, b_dims):
    y = (ctypes.c_int64 * 16)()
    r = ctypes.c_int(0)
    _check(_lib.onnx_matmul_infer(dims(a_dims), len(a_dims), dims(b_dims), len(b_dims), y, ctypes.byref(r)))
    return tuple(y[i] for i in range(r.value))


def onnx_conv(X, W, B=None, pads=(0, 0, 0, 0), strides=(1, 1), dilations=(1, 1), group=1,
              residual=None, act=ACT_NONE, out=None, stream=None):
    X, W, B, residual = _dev(X, "X"), _dev(W, "W"), _dev(B, "B"), _dev(residual, "residual")
    yd = onnx_conv_infer(X.shape, W.shape, pads, strides, dilations, group)
    Y = torch.empty(yd, dtype=torch.float32, device=X.device) if out is None else _dev(out, "out")
    _check(_lib.onnx_conv(_ptr(X), dims(X.shape), _ptr(W), dims(W.shape), _ptr(B), dims(pads),
                          dims(strides), dims(dilations), int(group), _ptr(residual), int(act), _ptr(Y),
                          dims(Y.shape), _stream(stream)))
    return Y


def onnx_conv_fixed_scratch(X, W, B=None, pads=(0, 0, 0, 0), strides=(1, 1), dilations=(1, 1), group=1,
                            residual=None, act=ACT_NONE, out=None, stream=None):
    """onnx_conv with the library's fixed split-K scratch.  The library call itself allocates nothing;
    pass ``out=`` to keep this wrapper from allocating the result."""
    X, W, B, residual = _dev(X, "X"), _dev(W, "W"), _dev(B, "B"), _dev(residual, "residual")
    yd = onnx_conv_infer(X.shape, W.shape, pads, strides, dilations, group)
    Y = torch.empty(yd, dtype=torch.float32, device=X.device) if out is None else _dev(out, "out")
    _check(_lib.onnx_conv_fixed_scratch(_ptr(X), dims(X.shape), _ptr(W), dims(W.shape), _ptr(B), dims(pads),
                                        dims(strides), dims(dilations), int(group), _ptr(residual), int(act),
                                        _ptr(Y), dims(Y.shape), _stream(stream)))
    return Y


def onnx_gemm(A, B, C=None, alpha=1.0, beta=1.0, transA=0, transB=0, act=ACT_NONE, out=None, stream=None):
    A, B, C = _dev(A, "A"), _dev(B, "B"), _dev(C, "C")
    M = A.shape[1] if transA else A.shape[0]
    N = B.shape[0] if transB else B.shape[1]
    Y = torch.empty((M, N), dtype=torch.float32, device=A.device) if out is None else _dev(out, "out")
    cd, cr = (dims(C.shape), C.dim()) if C is not None else (None, 0)
    _check(_lib.onnx_gemm(_ptr(A), dims(A.shape), _ptr(B), dims(B.shape), _ptr(C), cd, cr, float(alpha),
                          float(beta), int(transA), int(transB), int(act), _ptr(Y), dims(Y.shape),
                          _stream(stream)))
    return Y


def onnx_matmul(A, B, out=None, stream=None):
    A, B = _dev(A, "A"), _dev(B, "B")
    yd = onnx_matmul_infer(A.shape, B.shape)
    Y = torch.empty(yd, dtype=torch.float32, device=A.device) if out is None else _dev(out, "out")
    _check(_lib.onnx_matmul(_ptr(A), dims(A.shape), A.dim(), _ptr(B), dims(B.shape), B.dim(), _ptr(Y),
                            dims(Y.shape), Y.dim(), _stream(stream)))
    return Y


def onnx_maxpool(X, kernel, pads=(0, 0, 0, 0), strides=(1, 1), dilations=(1, 1), ceil_mode=0,
                 want_indices=False, out=None, out_indices=None, stream=None):
    X = _dev(X, "X")
    yd = onnx_pool_infer(X.shape, kernel, pads, strides, dilations, ceil_mode)
    Y = torch.empty(yd, dtype=torch.float32, device=X.device) if out is None else _dev(out, "out")
    I = out_indices
    if I is None and want_indices:
        I = torch.empty(yd, dtype=torch.int64, device=X.device)
    if I is not None and not (I.is_cuda and I.dtype == torch.int64 and I.is_contiguous()):
        raise TypeError("indices must be a contiguous int64 tensor on the GPU")
    _check(_lib.onnx_maxpool(_ptr(X), dims(X.shape), dims(kernel), dims(pads), dims(strides),
                             dims(dilations), int(ceil_mode), _ptr(Y), _ptr(I), dims(Y.shape),
                             _stream(stream)))
    return (Y, I) if I is not None else Y


def onnx_avgpool(X, kernel=None, pads=(0, 0, 0, 0), strides=(1, 1), ceil_mode=0, count_include_pad=0,
                 out=None, stream=None):
    X = _dev(X, "X")
    if kernel is None:
        yd = (X.shape[0], X.shape[1], 1, 1)
        kp = pp = sp = None
    else:
        yd = onnx_pool_infer(X.shape, kernel, pads, strides, (1, 1), ceil_mode)
        kp, pp, sp = dims(kernel), dims(pads), dims(strides)
    Y = torch.empty(yd, dtype=torch.float32, device=X.device) if out is None else _dev(out, "out")
    _check(_lib.onnx_avgpool(_ptr(X), dims(X.shape), kp, pp, sp, int(ceil_mode), int(count_include_pad),
                             _ptr(Y), dims(Y.shape), _stream(stream)))
    return Y


def onnx_broadcast_infer(a_dims, b_dims):
    y = (ctypes.c_int64 * 16)()
    r = ctypes.c_int(0)
    _check(_lib.onnx_broadcast_infer(dims(a_dims), len(a_dims), dims(b_dims), len(b_dims), y, ctypes.byref(r)))
    return tuple(y[i] for i in range(r.value))


def onnx_reduce_infer(x_dims, axes=None, keepdims=1):
    axes = [] if axes is None else list(axes)
    y = (ctypes.c_int64 * 16)()
    r = ctypes.c_int(0)
    _check(_lib.onnx_reduce_infer(dims(x_dims), len(x_dims), dims(axes), len(axes), int(keepdims), y, ctypes.byref(r)))
    return tuple(y[i] for i in range(r.value))


def _out(out, shape, like):
    return torch.empty(tuple(shape), dtype=torch.float32, device=like.device) if out is None else _dev(out, "out")


def onnx_add(A, B, out=None, stream=None):
    A, B = _dev(A, "A"), _dev(B, "B")
    Y = _out(out, onnx_broadcast_infer(A.shape, B.shape), A)
    _check(_lib.onnx_add(_ptr(A), dims(A.shape), A.dim(), _ptr(B), dims(B.shape), B.dim(), _ptr(Y), dims(Y.shape),
                         Y.dim(), _stream(stream)))
    return Y


def onnx_relu(X, out=None, stream=None):
    X = _dev(X, "X")
    Y = _out(out, X.shape, X)
    _check(_lib.onnx_relu(_ptr(X), X.numel(), _ptr(Y), _stream(stream)))
    return Y


def onnx_leakyrelu(X, alpha=0.01, out=None, stream=None):
    X = _dev(X, "X")
    Y = _out(out, X.shape, X)
    _check(_lib.onnx_leakyrelu(_ptr(X), X.numel(), float(alpha), _ptr(Y), _stream(stream)))
    return Y


def onnx_abs(X, out=None, stream=None):
    X = _dev(X, "X")
    Y = _out(out, X.shape, X)
    _check(_lib.onnx_abs(_ptr(X), X.numel(), _ptr(Y), _stream(stream)))
    return Y


def onnx_reducesum(X, axes=None, keepdims=1, out=None, stream=None):
    X = _dev(X, "X")
    axes = [] if axes is None else list(axes)
    Y = _out(out, onnx_reduce_infer(X.shape, axes, keepdims), X)
    _check(_lib.onnx_reducesum(_ptr(X), dims(X.shape), X.dim(), dims(axes), len(axes), int(keepdims), _ptr(Y),
                               dims(Y.shape), Y.dim(), _stream(stream)))
    return Y


def onnx_softmax(X, axis=-1, out=None, stream=None):
    X = _dev(X, "X")
    Y = _out(out, X.shape, X)
    _check(_lib.onnx_softmax(_ptr(X), dims(X.shape), X.dim(), int(axis), _ptr(Y), _stream(stream)))
    return Y


_LP_TYPES = {torch.float16: F16, torch.bfloat16: BF16}


def onnx_gemm_lp(A, B, C=None, alpha=1.0, beta=1.0, transA=0, transB=1, act=ACT_NONE, out_dtype=None, out=None,
                 stream=None):
    """Gemm on float16 / bfloat16 CUDA tensors (A [M,K], B [N,K] with transB=1), fp32 bias C, result in
    ``out_dtype`` (torch.float32 or the inputs' type; default the inputs' type, as ONNX Gemm does)."""
    if not (isinstance(A, torch.Tensor) and isinstance(B, torch.Tensor) and A.is_cuda and B.is_cuda and
            A.dtype == B.dtype and A.dtype in _LP_TYPES and A.is_contiguous() and B.is_contiguous()):
        raise TypeError("A and B must be contiguous float16 or bfloat16 tensors of one type on the GPU")
    C = _dev(C, "C")
    out_dtype = A.dtype if out_dtype is None else out_dtype
    if out_dtype not in (torch.float32, A.dtype):
        raise TypeError("out_dtype must be torch.float32 or the inputs' type")
    m = A.shape[1] if transA else A.shape[0]
    n = B.shape[0] if transB else B.shape[1]
    if out is None:
        out = torch.empty((m, n), dtype=out_dtype, device=A.device)
    elif not (out.is_cuda and out.dtype == out_dtype and out.is_contiguous()):
        raise TypeError("out must be a contiguous GPU tensor of out_dtype")
    cd, cr = (dims(C.shape), C.dim()) if C is not None else (None, 0)
    _check(_lib.onnx_gemm_lp(_ptr(A), dims(A.shape), _ptr(B), dims(B.shape), _ptr(C), cd, cr, float(alpha), float(beta),
                             int(transA), int(transB), int(act), _ptr(out), dims(out.shape), _LP_TYPES[A.dtype],
                             F32 if out_dtype == torch.float32 else _LP_TYPES[A.dtype], _stream(stream)))
    return out


def _lp(t, name, like=None):
    if t is None:
        return None
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype in _LP_TYPES and t.is_contiguous()):
        raise TypeError("%s must be a contiguous float16 or bfloat16 tensor on the GPU" % name)
    if like is not None and t.dtype != like.dtype:
        raise TypeError("%s must have the type of the other 16-bit operands" % name)
    return t


def _lp_out(out, shape, out_dtype, like):
    out_dtype = like.dtype if out_dtype is None else out_dtype
    if out_dtype not in (torch.float32, like.dtype):
        raise TypeError("out_dtype must be torch.float32 or the inputs' type")
    if out is None:
        out = torch.empty(tuple(shape), dtype=out_dtype, device=like.device)
    elif not (out.is_cuda and out.dtype == out_dtype and out.is_contiguous()):
        raise TypeError("out must be a contiguous GPU tensor of out_dtype")
    return out, (F32 if out_dtype == torch.float32 else _LP_TYPES[like.dtype])


def onnx_matmul_lp(A, B, out_dtype=None, out=None, stream=None):
    """MatMul on float16 / bfloat16 CUDA tensors, result in ``out_dtype`` (default: the inputs' type)."""
    A = _lp(A, "A")
    B = _lp(B, "B", A)
    Y, ot = _lp_out(out, onnx_matmul_infer(A.shape, B.shape), out_dtype, A)
    _check(_lib.onnx_matmul_lp(_ptr(A), dims(A.shape), A.dim(), _ptr(B), dims(B.shape), B.dim(), _ptr(Y), dims(Y.shape),
                               Y.dim(), _LP_TYPES[A.dtype], ot, _stream(stream)))
    return Y


def onnx_conv_lp(X, W, B=None, pads=(0, 0, 0, 0), strides=(1, 1), dilations=(1, 1), group=1, residual=None,
                 act=ACT_NONE, out_dtype=None, out=None, stream=None):
    """Conv on float16 / bfloat16 CUDA tensors X, W; fp32 bias B; result (and residual) in ``out_dtype``."""
    X = _lp(X, "X")
    W = _lp(W, "W", X)
    B = _dev(B, "B")
    Y, ot = _lp_out(out, onnx_conv_infer(X.shape, W.shape, pads, strides, dilations, group), out_dtype, X)
    if residual is not None and not (residual.is_cuda and residual.dtype == Y.dtype and residual.is_contiguous()):
        raise TypeError("residual must be a contiguous GPU tensor of the result's type")
    _check(_lib.onnx_conv_lp(_ptr(X), dims(X.shape), _ptr(W), dims(W.shape), _ptr(B), dims(pads), dims(strides),
                             dims(dilations), int(group), _ptr(residual), int(act), _ptr(Y), dims(Y.shape),
                             _LP_TYPES[X.dtype], ot, _stream(stream)))
    return Y


def onnx_conv_lp_filter_taps(W, stream=None):
    """A 3x3 filter bank [M, C/group, 3, 3] (C/group a multiple of 16) rewritten into the tap order onnx_conv_lp_taps reads."""
    W = _lp(W, "W")
    packed = torch.empty_like(W)
    _check(_lib.onnx_conv_lp_filter_taps(_ptr(W), dims(W.shape), _ptr(packed), _stream(stream)))
    return packed


def onnx_conv_lp_taps(X, packed, B=None, pads=(0, 0, 0, 0), strides=(1, 1), dilations=(1, 1), group=1, residual=None,
                      act=ACT_NONE, out_dtype=None, out=None, stream=None):
    """onnx_conv_lp for a 3x3 filter bank rewritten by onnx_conv_lp_filter_taps (it keeps W's shape); needs no workspace."""
    X = _lp(X, "X")
    packed = _lp(packed, "packed", X)
    B = _dev(B, "B")
    Y, ot = _lp_out(out, onnx_conv_infer(X.shape, packed.shape, pads, strides, dilations, group), out_dtype, X)
    if residual is not None and not (residual.is_cuda and residual.dtype == Y.dtype and residual.is_contiguous()):
        raise TypeError("residual must be a contiguous GPU tensor of the result's type")
    _check(_lib.onnx_conv_lp_taps(_ptr(X), dims(X.shape), _ptr(packed), dims(packed.shape), _ptr(B), dims(pads), dims(strides),
                                  dims(dilations), int(group), _ptr(residual), int(act), _ptr(Y), dims(Y.shape),
                                  _LP_TYPES[X.dtype], ot, _stream(stream)))
    return Y


def onnx_leakyrelu_lp(X, alpha=0.01, out=None, stream=None):
    """LeakyRelu on a float16 / bfloat16 CUDA tensor (alpha = 0: Relu); the result has the same type."""
    X = _lp(X, "X")
    Y, _ = _lp_out(out, X.shape, X.dtype, X)
    _check(_lib.onnx_leakyrelu_lp(_ptr(X), X.numel(), float(alpha), _ptr(Y), _LP_TYPES[X.dtype], _stream(stream)))
    return Y


def onnx_add_lp(A, B, out=None, stream=None):
    """Add with numpy-style broadcasting on two float16 / bfloat16 CUDA tensors of one type; the result has that type."""
    A, B = _lp(A, "A"), _lp(B, "B")
    if A.dtype != B.dtype:
        raise TypeError("A and B must have the same 16-bit type")
    Y, _ = _lp_out(out, onnx_broadcast_infer(A.shape, B.shape), A.dtype, A)
    _check(_lib.onnx_add_lp(_ptr(A), dims(A.shape), A.dim(), _ptr(B), dims(B.shape), B.dim(), _ptr(Y), dims(Y.shape),
                            Y.dim(), _LP_TYPES[A.dtype], _stream(stream)))
    return Y


def onnx_abs_lp(X, out=None, stream=None):
    """Abs on a float16 / bfloat16 CUDA tensor; the result has the same type."""
    X = _lp(X, "X")
    Y, _ = _lp_out(out, X.shape, X.dtype, X)
    _check(_lib.onnx_abs_lp(_ptr(X), X.numel(), _ptr(Y), _LP_TYPES[X.dtype], _stream(stream)))
    return Y


def onnx_reducesum_lp(X, axes=None, keepdims=1, out=None, stream=None):
    """ReduceSum on a float16 / bfloat16 CUDA tensor (fp32 sums); the result has the same type."""
    X = _lp(X, "X")
    axes = [] if axes is None else list(axes)
    Y, _ = _lp_out(out, onnx_reduce_infer(X.shape, axes, keepdims), X.dtype, X)
    _check(_lib.onnx_reducesum_lp(_ptr(X), dims(X.shape), X.dim(), dims(axes), len(axes), int(keepdims), _ptr(Y),
                                  dims(Y.shape), Y.dim(), _LP_TYPES[X.dtype], _stream(stream)))
    return Y


def onnx_softmax_lp(X, axis=-1, out=None, stream=None):
    """Softmax on a float16 / bfloat16 CUDA tensor (fp32 arithmetic); the result has the same type."""
    X = _lp(X, "X")
    Y, _ = _lp_out(out, X.shape, X.dtype, X)
    _check(_lib.onnx_softmax_lp(_ptr(X), dims(X.shape), X.dim(), int(axis), _ptr(Y), _LP_TYPES[X.dtype], _stream(stream)))
    return Y


def onnx_maxpool_lp(X, kernel, pads=(0, 0, 0, 0), strides=(1, 1), dilations=(1, 1), ceil_mode=0, out=None, stream=None):
    """MaxPool on a float16 / bfloat16 CUDA tensor; the result has the same type."""
    X = _lp(X, "X")
    Y, _ = _lp_out(out, onnx_pool_infer(X.shape, kernel, pads, strides, dilations, ceil_mode), X.dtype, X)
    _check(_lib.onnx_maxpool_lp(_ptr(X), dims(X.shape), dims(kernel), dims(pads), dims(strides), dims(dilations),
                                int(ceil_mode), _ptr(Y), dims(Y.shape), _LP_TYPES[X.dtype], _stream(stream)))
    return Y


def onnx_avgpool_lp(X, kernel=None, pads=(0, 0, 0, 0), strides=(1, 1), ceil_mode=0, count_include_pad=0, out=None,
                    stream=None):
    """AveragePool (kernel=None: GlobalAveragePool) on a float16 / bfloat16 CUDA tensor; the result has the same type."""
    X = _lp(X, "X")
    if kernel is None:
        yd = (X.shape[0], X.shape[1], 1, 1)
        kp = pp = sp = None
    else:
        yd = onnx_pool_infer(X.shape, kernel, pads, strides, (1, 1), ceil_mode)
        kp, pp, sp = dims(kernel), dims(pads), dims(strides)
    Y, _ = _lp_out(out, yd, X.dtype, X)
    _check(_lib.onnx_avgpool_lp(_ptr(X), dims(X.shape), kp, pp, sp, int(ceil_mode), int(count_include_pad),
                                _ptr(Y), dims(Y.shape), _LP_TYPES[X.dtype], _stream(stream)))
    return Y


def onnx_lstm(X, W, R, B=None, initial_h=None, initial_c=None, direction="forward", stream=None):
    """ONNX LSTM (layout 0, default activations).  Returns (Y, Y_h, Y_c); the scratch the library
    needs is allocated here with torch.empty and lives until the call's work has been enqueued
    (torch keeps the block alive for the stream it was allocated on)."""
    X, W, R = _dev(X, "X"), _dev(W, "W"), _dev(R, "R")
    B, initial_h, initial_c = _dev(B, "B"), _dev(initial_h, "initial_h"), _dev(initial_c, "initial_c")
    d = LSTM_DIRECTIONS[direction]
    dirs = 2 if d == 2 else 1
    seq, batch, _ = X.shape
    H = R.shape[2]
    if tuple(W.shape) != (dirs, 4 * H, X.shape[2]) or tuple(R.shape) != (dirs, 4 * H, H):
        raise ValueError("W must be [dirs, 4H, input] and R [dirs, 4H, H]")
    for t, shape, name in ((B, (dirs, 8 * H), "B"), (initial_h, (dirs, batch, H), "initial_h"), (initial_c, (dirs, batch, H), "initial_c")):
        if t is not None and tuple(t.shape) != shape:
            raise ValueError("%s must have shape %r" % (name, shape))
    Y = torch.empty((seq, dirs, batch, H), dtype=torch.float32, device=X.device)
    Yh = torch.empty((dirs, batch, H), dtype=torch.float32, device=X.device)
    Yc = torch.empty((dirs, batch, H), dtype=torch.float32, device=X.device)
    need = _lib.onnx_lstm_scratch_bytes(dims(X.shape), H, d)
    scratch = torch.empty(max(need, 256), dtype=torch.uint8, device=X.device)
    _check(_lib.onnx_lstm(_ptr(X), dims(X.shape), _ptr(W), _ptr(R), _ptr(B), _ptr(initial_h), _ptr(initial_c), H, d,
                          _ptr(Y), _ptr(Yh), _ptr(Yc), _ptr(scratch), scratch.numel(), _stream(stream)))
    return Y, Yh, Yc


CHAIN_KINDS = {"conv": 0, "maxpool": 1, "avgpool": 2, "gemm": 3}
CHAIN_MAX_OPS = 8
CHAIN_MAX_ACTIVATION = 10240
CHAIN_MAX_WEIGHTS = 14336
CHAIN_MAX_CONV_K = 2048


def chain_shapes(x_dims, ops):
    """Result shape of every operator of a chain (host only; the library's *_infer calls)."""
    d = tuple(int(v) for v in x_dims)
    shapes = []
    for o in ops:
        kind = o["op"]
        if kind == "conv":
            w = o["W"].shape
            d = onnx_conv_infer(d, (w[0], d[1], w[2], w[3]), o.get("pads", (0, 0, 0, 0)), o.get("strides", (1, 1)),
                                o.get("dilations", (1, 1)), 1)
        elif kind == "maxpool":
            d = onnx_pool_infer(d, o["kernel"], o.get("pads", (0, 0, 0, 0)), o.get("strides", (1, 1)),
                                o.get("dilations", (1, 1)), o.get("ceil_mode", 0))
        elif kind == "avgpool":
            if o.get("kernel") is None:
                d = (d[0], d[1], 1, 1)
            else:
                d = onnx_pool_infer(d, o["kernel"], o.get("pads", (0, 0, 0, 0)), o.get("strides", (1, 1)), (1, 1),
                                    o.get("ceil_mode", 0))
        elif kind == "gemm":
            w = o["W"].shape
            d = (d[0], int(w[0] if o.get("transB", 0) else w[1]), 1, 1)
        else:
            raise ValueError("unknown chain operator %r" % kind)
        shapes.append(tuple(d))
    return shapes


def onnx_chain_args(X, ops, keep=False, outs=None):
    """Marshals a chain into the C structures: returns (array of onnx_chain_op, result tensors).
    ``ops`` is a list of dicts: {"op": "conv", "W", "B", "pads", "strides", "dilations", "act"},
    {"op": "maxpool", "kernel", "pads", "strides", "dilations", "ceil_mode"}, {"op": "avgpool",
    "kernel" (None = global), "pads", "strides", "ceil_mode", "count_include_pad"}, {"op": "gemm",
    "W", "B", "transB", "alpha", "beta", "act"}.  With ``keep`` every operator's result is
    written to device memory, otherwise only the last one's; a Gemm's result is [N, outputs]."""
    X = _dev(X, "X")
    shapes = chain_shapes(X.shape, ops)
    arr = (ChainOp * max(len(ops), 1))()
    results = []
    for i, (o, shp) in enumerate(zip(ops, shapes)):
        c = arr[i]
        c.kind = CHAIN_KINDS[o["op"]]
        c.act = int(o.get("act", ACT_NONE))
        W, B = _dev(o.get("W"), "W"), _dev(o.get("B"), "B")
        c.outputs = shp[1] if o["op"] in ("conv", "gemm") else 0
        k = o.get("kernel") if o["op"] != "conv" else W.shape[2:]
        c.kernel[0], c.kernel[1] = (0, 0) if k is None else (int(k[0]), int(k[1]))
        for j, v in enumerate(o.get("pads", (0, 0, 0, 0))): c.pads[j] = int(v)
        for j, v in enumerate(o.get("strides", (1, 1))): c.strides[j] = int(v)
        for j, v in enumerate(o.get("dilations", (1, 1))): c.dilations[j] = int(v)
        c.ceil_mode = int(o.get("ceil_mode", 0))
        c.count_include_pad = int(o.get("count_include_pad", 0))
        c.transB = int(o.get("transB", 0))
        c.alpha, c.beta = float(o.get("alpha", 1.0)), float(o.get("beta", 1.0))
        c.W = None if W is None else W.data_ptr()
        c.B = None if B is None else B.data_ptr()
        y = None
        if keep or i == len(ops) - 1:
            out_shape = (shp[0], shp[1]) if o["op"] == "gemm" else shp
            y = outs[i] if outs is not None and outs[i] is not None else torch.empty(out_shape, dtype=torch.float32, device=X.device)
            y = _dev(y, "out")
        c.Y = None if y is None else y.data_ptr()
        results.append(y)
    return arr, results


def onnx_chain(X, ops, keep=False, outs=None, stream=None):
    """A linear chain of Conv / MaxPool / AveragePool / Gemm operators in one launch (see
    onnx_chain_args for ``ops``).  Returns the last result, or with ``keep`` the list of all."""
    X = _dev(X, "X")
    arr, results = onnx_chain_args(X, ops, keep, outs)
    _check(_lib.onnx_chain(arr, len(ops), _ptr(X), dims(X.shape), _stream(stream)))
    return results if keep else results[-1]
