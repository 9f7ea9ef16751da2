"""Runs a workload graph with the CPU oracle (test infrastructure only).

Graphs may be in the fused form the GPU runner executes or in the operator-by-operator form
an exporter writes (BatchNormalization, Relu, Add, Identity, MatMul as nodes of their own: the
inputs of the graph-level passes of Section 3.4 of the paper); the latter are evaluated by
their definitions, so a rewritten graph can be checked against the graph it came from.

Each node is evaluated by the oracle in double precision from fp32 inputs; the
result is rounded to fp32 once, when it is handed to the next node, as a chain
of fp32 operators would store it.  ``run`` returns every fp32 activation and the
un-rounded double result of each node, so a test can compare any layer.
"""
import numpy as np

from . import avgpool, conv, gemm, matmul, maxpool
from . import elementwise as ew


def batchnorm(x, scale, bias, mean, var, eps):
    """ONNX BatchNormalization at inference, per channel c of an N x C x ... tensor, in double:
    y = (x - mean[c]) / sqrt(var[c] + eps) * scale[c] + bias[c]."""
    x = np.asarray(x, dtype=np.float64)
    shp = (1, -1) + (1,) * (x.ndim - 2)
    f = lambda v: np.asarray(v, dtype=np.float64).reshape(shp)
    return (x - f(mean)) / np.sqrt(f(var) + float(eps)) * f(scale) + f(bias)


def run(model, keep=None):
    env = {}
    env.update(model["inputs"])
    env.update(model["weights"])
    exact = {}
    for nd in model["graph"]:
        op = nd["op"]
        if op == "conv":
            res = env[nd["residual"]] if nd["residual"] else None
            b = env[nd["b"]] if nd["b"] else None
            y = conv(env[nd["x"]], env[nd["w"]], b, nd["pads"], nd["strides"], nd["dilations"],
                     nd["group"], residual=res, relu=nd["relu"])
        elif op == "maxpool":
            y = maxpool(env[nd["x"]], nd["kernel"], nd["pads"], nd["strides"], nd["dilations"],
                        nd["ceil_mode"], want_indices=False)
        elif op == "avgpool":
            y = avgpool(env[nd["x"]], nd["kernel"], nd["pads"], nd["strides"], nd["ceil_mode"],
                        nd["count_include_pad"])
        elif op == "reshape":
            y = np.reshape(env[nd["x"]], nd["shape"])
        elif op == "gemm":
            c = env[nd["c"]] if nd["c"] else None
            y = gemm(env[nd["a"]], env[nd["b"]], c, nd["alpha"], nd["beta"], nd["transA"],
                     nd["transB"], relu=nd["relu"])
        elif op == "matmul":
            y = matmul(env[nd["a"]], env[nd["b"]])
        elif op == "batchnorm":
            y = batchnorm(env[nd["x"]], env[nd["scale"]], env[nd["bias"]], env[nd["mean"]],
                          env[nd["var"]], nd["eps"])
        elif op == "relu":
            y = ew.relu(env[nd["x"]])
        elif op == "add":
            y = ew.add(env[nd["a"]], env[nd["b"]])
        elif op == "leakyrelu":
            y = ew.leakyrelu(env[nd["x"]], nd["alpha"])
        elif op == "abs":
            y = ew.absolute(env[nd["x"]])
        elif op == "reducesum":
            y = ew.reducesum(env[nd["x"]], nd["axes"], nd["keepdims"])
        elif op == "reducel1":
            y = ew.reducel1(env[nd["x"]], nd["axes"], nd["keepdims"])
        elif op == "softmax":
            y = ew.softmax(env[nd["x"]], nd["axis"])
        elif op == "identity":
            y = np.asarray(env[nd["x"]], dtype=np.float64)
        else:
            raise ValueError("unknown node op %r" % (op,))
        if keep is None or nd["y"] in keep or nd["y"] == model["output"]:
            exact[nd["y"]] = y
        env[nd["y"]] = np.asarray(y, dtype=np.float32)
    return env, exact
