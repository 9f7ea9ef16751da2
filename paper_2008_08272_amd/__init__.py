"""ONNX Conv / Gemm / MatMul / MaxPool / AveragePool (and the element-wise, ReduceSum, Softmax, LSTM
and 16-bit Gemm operators around them) on one MI355X (gfx950).

The operators run in hand-written HIP kernels behind a C-ABI library (``libonnxhip.so``,
declared in ``include/onnxhip.h``).  This package is the thin Python binding: it marshals
torch device tensors into that ABI.  There is no CPU or PyTorch fallback: if the library has
not been built, the first use of any operator raises ImportError.

The binding is loaded on first use, so that ``paper_2008_08272_amd.build`` (which produces the
library) can be imported before the library exists.
"""
import importlib

_BINDING_NAMES = (
    "OnnxHipError", "lib_path", "onnx_chain", "chain_shapes", "onnx_abs", "onnx_add", "onnx_avgpool", "onnx_broadcast_infer", "onnx_conv",
    "onnx_conv_fixed_scratch", "onnx_conv_lp", "onnx_conv_lp_taps", "onnx_conv_lp_filter_taps", "onnx_maxpool_lp", "onnx_leakyrelu_lp", "onnx_add_lp", "onnx_abs_lp", "onnx_reducesum_lp", "onnx_softmax_lp", "onnx_avgpool_lp", "onnx_last_launch", "onnx_matmul_lp",
    "onnx_conv_infer", "onnx_gemm", "onnx_gemm_lp", "onnx_last_error", "onnx_leakyrelu", "onnx_lstm", "onnx_matmul",
    "onnx_matmul_infer", "onnx_maxpool", "onnx_pool_infer", "onnx_reduce_infer", "onnx_reducesum", "onnx_relu",
    "onnx_set_workspace", "onnx_softmax",
)


def __getattr__(name):
    if name in _BINDING_NAMES:
        return getattr(importlib.import_module(".binding", __name__), name)
    raise AttributeError("module %r has no attribute %r" % (__name__, name))


def __dir__():
    return sorted(list(globals()) + list(_BINDING_NAMES))
