"""ONNX Conv / Gemm / MatMul / MaxPool / AveragePool (and the element-wise, ReduceSum and Softmax
operators around them) on one MI355X (gfx950).

The operators run in hand-written HIP kernels behind a C-ABI library (``libonnxhip.so``,
declared in ``include/onnxhip.h``).  This package is the thin Python binding: it marshals
torch device tensors into that ABI.  There is no CPU or PyTorch fallback: if the library has
not been built, importing :mod:`paper_2008_08272_amd.binding` raises.
"""
from .binding import (OnnxHipError, lib_path, onnx_avgpool, onnx_conv, onnx_conv_infer, onnx_gemm,  # noqa: F401
                      onnx_last_error, onnx_matmul, onnx_set_workspace, onnx_matmul_infer, onnx_maxpool, onnx_pool_infer,
                      onnx_abs, onnx_add, onnx_broadcast_infer, onnx_leakyrelu, onnx_reduce_infer, onnx_reducesum,
                      onnx_relu, onnx_softmax, onnx_gemm_lp)
