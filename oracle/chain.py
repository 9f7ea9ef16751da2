"""Runs a workload graph with the CPU oracle (test infrastructure only).

Each node is evaluated by the oracle in double precision from fp32 inputs; the
result is rounded to fp32 once, when it is handed to the next node, as a chain
of fp32 operators would store it.  ``run`` returns every fp32 activation and the
un-rounded double result of each node, so a test can compare any layer.
"""
import numpy as np

from . import avgpool, conv, gemm, matmul, maxpool


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
        else:
            raise ValueError("unknown node op %r" % (op,))
        if keep is None or nd["y"] in keep or nd["y"] == model["output"]:
            exact[nd["y"]] = y
        env[nd["y"]] = np.asarray(y, dtype=np.float32)
    return env, exact
