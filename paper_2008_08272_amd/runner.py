"""Tiny model runner: chains library calls for a workload graph.

The analogue of the single entry function a compiled model exports in the paper (Section 3):
the graph's constant inputs are uploaded once, every activation buffer is allocated once, and
``run()`` enqueues one library call per node on one stream with no host synchronisation in
between.  Reshape is a view of dense row-major data and costs nothing.  A model that is one
linear chain of Conv / pool / Gemm nodes small enough for the library's single-launch chain
(``onnx_chain``: every activation and all weights in LDS) is run through that one call
instead.  All arithmetic happens inside the library's kernels; this module only prepares
argument lists.

With ``dtype=torch.float16`` or ``torch.bfloat16`` a graph of Conv / MaxPool / AveragePool / Reshape /
Gemm / MatMul / Relu / LeakyRelu nodes runs on 16-bit tensors (the operator definitions admit them, Section 3.1):
inputs and weights are rounded to the type once, on upload, the biases stay fp32, every
activation is stored in the type (fp32 accumulation inside each operator), and the node that
produces the model's output stores fp32.
"""

import numpy as np
import torch

from . import binding as B


class GraphRunner:
    def __init__(self, model, device="cuda:0", workspace_bytes=64 << 20, fuse_chain=True, keep_intermediates=False,
                 dtype=None):
        """fuse_chain: use the single-launch chain when the model qualifies.  keep_intermediates:
        have the chain write every node's result to device memory too (for layer-by-layer checks;
        the per-node path always does).  dtype: None (fp32) or the 16-bit type to run in."""
        self.device = torch.device(device)
        self.model = model
        self.dtype = None if dtype in (None, torch.float32) else dtype
        if self.dtype is not None:
            self._init_lp(workspace_bytes)
            return
        for nd in model["graph"]:                  # refuse before anything is allocated or registered
            if nd["op"] in ("batchnorm", "identity", "reducel1"):
                raise NotImplementedError(
                    "node %r (%s) has no kernel of its own: run paper_2008_08272_amd.passes.optimize on the "
                    "graph first; it folds, removes or decomposes such nodes" % (nd["y"], nd["op"]))
        # scratch the library may use to split the K range of products with few output tiles
        # (set as the library's workspace at the start of every run)
        self.workspace = None
        if workspace_bytes:
            self.workspace = torch.empty(workspace_bytes, dtype=torch.uint8, device=self.device)
        self.t = {}
        for k, v in list(model["inputs"].items()) + list(model["weights"].items()):
            self.t[k] = torch.from_numpy(np.ascontiguousarray(v, dtype=np.float32)).to(self.device)
        self.calls = []
        lib = B.raw()
        for nd in model["graph"]:
            op = nd["op"]
            if op == "conv":
                x, w = self.t[nd["x"]], self.t[nd["w"]]
                yd = B.onnx_conv_infer(x.shape, w.shape, nd["pads"], nd["strides"], nd["dilations"], nd["group"])
                y = self._new(nd["y"], yd)
                b = self.t[nd["b"]] if nd["b"] else None
                r = self.t[nd["residual"]] if nd["residual"] else None
                args = [B._ptr(x), B.dims(x.shape), B._ptr(w), B.dims(w.shape), B._ptr(b), B.dims(nd["pads"]),
                        B.dims(nd["strides"]), B.dims(nd["dilations"]), int(nd["group"]), B._ptr(r),
                        B.ACT_RELU if nd["relu"] else B.ACT_NONE, B._ptr(y), B.dims(y.shape), None]
                self.calls.append((lib.onnx_conv, args))
            elif op == "maxpool":
                x = self.t[nd["x"]]
                yd = B.onnx_pool_infer(x.shape, nd["kernel"], nd["pads"], nd["strides"], nd["dilations"], nd["ceil_mode"])
                y = self._new(nd["y"], yd)
                args = [B._ptr(x), B.dims(x.shape), B.dims(nd["kernel"]), B.dims(nd["pads"]), B.dims(nd["strides"]),
                        B.dims(nd["dilations"]), int(nd["ceil_mode"]), B._ptr(y), None, B.dims(y.shape), None]
                self.calls.append((lib.onnx_maxpool, args))
            elif op == "avgpool":
                x = self.t[nd["x"]]
                if nd["kernel"] is None:
                    yd = (x.shape[0], x.shape[1], 1, 1)
                    kp = pp = sp = None
                else:
                    yd = B.onnx_pool_infer(x.shape, nd["kernel"], nd["pads"], nd["strides"], (1, 1), nd["ceil_mode"])
                    kp, pp, sp = B.dims(nd["kernel"]), B.dims(nd["pads"]), B.dims(nd["strides"])
                y = self._new(nd["y"], yd)
                args = [B._ptr(x), B.dims(x.shape), kp, pp, sp, int(nd["ceil_mode"]), int(nd["count_include_pad"]),
                        B._ptr(y), B.dims(y.shape), None]
                self.calls.append((lib.onnx_avgpool, args))
            elif op == "reshape":
                self.t[nd["y"]] = self.t[nd["x"]].view(nd["shape"])
            elif op == "gemm":
                a, b = self.t[nd["a"]], self.t[nd["b"]]
                c = self.t[nd["c"]] if nd["c"] else None
                m = a.shape[1] if nd["transA"] else a.shape[0]
                n = b.shape[0] if nd["transB"] else b.shape[1]
                y = self._new(nd["y"], (m, n))
                cd, cr = (B.dims(c.shape), c.dim()) if c is not None else (None, 0)
                args = [B._ptr(a), B.dims(a.shape), B._ptr(b), B.dims(b.shape), B._ptr(c), cd, cr,
                        float(nd["alpha"]), float(nd["beta"]), int(nd["transA"]), int(nd["transB"]),
                        B.ACT_RELU if nd["relu"] else B.ACT_NONE, B._ptr(y), B.dims(y.shape), None]
                self.calls.append((lib.onnx_gemm, args))
            elif op == "matmul":
                a, b = self.t[nd["a"]], self.t[nd["b"]]
                yd = B.onnx_matmul_infer(a.shape, b.shape)
                y = self._new(nd["y"], yd)
                args = [B._ptr(a), B.dims(a.shape), a.dim(), B._ptr(b), B.dims(b.shape), b.dim(), B._ptr(y),
                        B.dims(y.shape), y.dim(), None]
                self.calls.append((lib.onnx_matmul, args))
            elif op == "add":
                a, b = self.t[nd["a"]], self.t[nd["b"]]
                y = self._new(nd["y"], B.onnx_broadcast_infer(a.shape, b.shape))
                args = [B._ptr(a), B.dims(a.shape), a.dim(), B._ptr(b), B.dims(b.shape), b.dim(), B._ptr(y),
                        B.dims(y.shape), y.dim(), None]
                self.calls.append((lib.onnx_add, args))
            elif op in ("relu", "abs", "leakyrelu"):
                x = self.t[nd["x"]]
                y = self._new(nd["y"], x.shape)
                if op == "leakyrelu":
                    self.calls.append((lib.onnx_leakyrelu, [B._ptr(x), x.numel(), float(nd["alpha"]), B._ptr(y), None]))
                else:
                    fn = lib.onnx_relu if op == "relu" else lib.onnx_abs
                    self.calls.append((fn, [B._ptr(x), x.numel(), B._ptr(y), None]))
            elif op == "reducesum":
                x = self.t[nd["x"]]
                axes = [] if nd["axes"] is None else list(nd["axes"])
                y = self._new(nd["y"], B.onnx_reduce_infer(x.shape, axes, nd["keepdims"]))
                args = [B._ptr(x), B.dims(x.shape), x.dim(), B.dims(axes), len(axes), int(nd["keepdims"]), B._ptr(y),
                        B.dims(y.shape), y.dim(), None]
                self.calls.append((lib.onnx_reducesum, args))
            elif op == "softmax":
                x = self.t[nd["x"]]
                y = self._new(nd["y"], x.shape)
                self.calls.append((lib.onnx_softmax, [B._ptr(x), B.dims(x.shape), x.dim(), int(nd["axis"]), B._ptr(y), None]))
            else:
                raise ValueError("unknown node op %r" % (op,))
        self.output = self.t[model["output"]]
        self.chain = self._build_chain(keep_intermediates) if fuse_chain else None

    def _init_lp(self, workspace_bytes):
        """The 16-bit form of the graph: the same nodes through the library's 16-bit entry points."""
        model, dt = self.model, self.dtype
        if dt not in (torch.float16, torch.bfloat16):
            raise TypeError("dtype must be torch.float32, torch.float16 or torch.bfloat16")
        code = B.F16 if dt == torch.float16 else B.BF16
        fp32_names = set()                         # the additive operands, which the 16-bit operators take in fp32
        for nd in model["graph"]:
            if nd["op"] not in ("conv", "maxpool", "avgpool", "reshape", "gemm", "matmul", "relu", "leakyrelu", "add", "abs", "reducesum",
                                "softmax"):
                raise NotImplementedError("node %r (%s): the 16-bit runner takes Conv, MaxPool, AveragePool, Reshape, Gemm, "
                                          "MatMul, Relu, LeakyRelu, Add, Abs, ReduceSum and Softmax nodes" % (nd["y"], nd["op"]))
            if nd["op"] == "conv" and nd["b"]:
                fp32_names.add(nd["b"])
            if nd["op"] == "gemm" and nd["c"]:
                fp32_names.add(nd["c"])
        self.workspace = torch.empty(workspace_bytes, dtype=torch.uint8, device=self.device) if workspace_bytes else None
        self.t = {}
        for k, v in list(model["inputs"].items()) + list(model["weights"].items()):
            t = torch.from_numpy(np.ascontiguousarray(v, dtype=np.float32)).to(self.device)
            self.t[k] = t if k in fp32_names else t.to(dt)
        self.calls = []
        self.chain = None
        lib = B.raw()
        for nd in model["graph"]:
            op = nd["op"]
            last = nd["y"] == model["output"]
            ydt, ycode = (torch.float32, B.F32) if last and op in ("conv", "gemm", "matmul") else (dt, code)
            if op == "conv":
                x, w = self.t[nd["x"]], self.t[nd["w"]]
                yd = B.onnx_conv_infer(x.shape, w.shape, nd["pads"], nd["strides"], nd["dilations"], nd["group"])
                y = self._new(nd["y"], yd, ydt)
                b = self.t[nd["b"]] if nd["b"] else None
                r = self.t[nd["residual"]] if nd["residual"] else None
                if r is not None and r.dtype != ydt:
                    raise NotImplementedError("node %r: a residual must have the type of the result" % (nd["y"],))
                args = [B._ptr(x), B.dims(x.shape), B._ptr(w), B.dims(w.shape), B._ptr(b), B.dims(nd["pads"]),
                        B.dims(nd["strides"]), B.dims(nd["dilations"]), int(nd["group"]), B._ptr(r),
                        B.ACT_RELU if nd["relu"] else B.ACT_NONE, B._ptr(y), B.dims(y.shape), code, ycode, None]
                fn = lib.onnx_conv_lp
                if tuple(w.shape[2:]) == (3, 3) and w.shape[1] % 16 == 0:
                    # the weights are constants: rewrite the filter bank into the 3x3 kernel's tap order once, here,
                    # instead of on every call; one untimed call finds out whether the kernel takes this shape
                    taps = B.onnx_conv_lp_filter_taps(w)
                    trial = list(args)
                    trial[2], trial[-1] = B._ptr(taps), B._stream(None)
                    st = lib.onnx_conv_lp_taps(*trial)
                    if st == B.ONNX_OK:
                        self.t[nd["w"] + ".taps"] = taps
                        args[2], fn = B._ptr(taps), lib.onnx_conv_lp_taps
                    elif st != B.ONNX_ERR_UNSUPPORTED:
                        raise B.OnnxHipError(st, B.onnx_last_error())
                self.calls.append((fn, args))
            elif op == "maxpool":
                x = self.t[nd["x"]]
                yd = B.onnx_pool_infer(x.shape, nd["kernel"], nd["pads"], nd["strides"], nd["dilations"], nd["ceil_mode"])
                y = self._new(nd["y"], yd, dt)
                args = [B._ptr(x), B.dims(x.shape), B.dims(nd["kernel"]), B.dims(nd["pads"]), B.dims(nd["strides"]),
                        B.dims(nd["dilations"]), int(nd["ceil_mode"]), B._ptr(y), B.dims(y.shape), code, None]
                self.calls.append((lib.onnx_maxpool_lp, args))
            elif op == "avgpool":
                x = self.t[nd["x"]]
                if nd["kernel"] is None:
                    yd = (x.shape[0], x.shape[1], 1, 1)
                    kp = pp = sp = None
                else:
                    yd = B.onnx_pool_infer(x.shape, nd["kernel"], nd["pads"], nd["strides"], (1, 1), nd["ceil_mode"])
                    kp, pp, sp = B.dims(nd["kernel"]), B.dims(nd["pads"]), B.dims(nd["strides"])
                y = self._new(nd["y"], yd, dt)
                args = [B._ptr(x), B.dims(x.shape), kp, pp, sp, int(nd["ceil_mode"]), int(nd["count_include_pad"]),
                        B._ptr(y), B.dims(y.shape), code, None]
                self.calls.append((lib.onnx_avgpool_lp, args))
            elif op == "reshape":
                self.t[nd["y"]] = self.t[nd["x"]].view(nd["shape"])
            elif op == "gemm":
                a, b = self.t[nd["a"]], self.t[nd["b"]]
                c = self.t[nd["c"]] if nd["c"] else None
                m = a.shape[1] if nd["transA"] else a.shape[0]
                n = b.shape[0] if nd["transB"] else b.shape[1]
                y = self._new(nd["y"], (m, n), ydt)
                cd, cr = (B.dims(c.shape), c.dim()) if c is not None else (None, 0)
                args = [B._ptr(a), B.dims(a.shape), B._ptr(b), B.dims(b.shape), B._ptr(c), cd, cr,
                        float(nd["alpha"]), float(nd["beta"]), int(nd["transA"]), int(nd["transB"]),
                        B.ACT_RELU if nd["relu"] else B.ACT_NONE, B._ptr(y), B.dims(y.shape), code, ycode, None]
                self.calls.append((lib.onnx_gemm_lp, args))
            elif op in ("relu", "leakyrelu"):
                x = self.t[nd["x"]]
                y = self._new(nd["y"], x.shape, dt)
                alpha = float(nd["alpha"]) if op == "leakyrelu" else 0.0
                self.calls.append((lib.onnx_leakyrelu_lp, [B._ptr(x), x.numel(), alpha, B._ptr(y), code, None]))
            elif op == "add":
                a, b = self.t[nd["a"]], self.t[nd["b"]]
                y = self._new(nd["y"], B.onnx_broadcast_infer(a.shape, b.shape), dt)
                args = [B._ptr(a), B.dims(a.shape), a.dim(), B._ptr(b), B.dims(b.shape), b.dim(), B._ptr(y),
                        B.dims(y.shape), y.dim(), code, None]
                self.calls.append((lib.onnx_add_lp, args))
            elif op == "abs":
                x = self.t[nd["x"]]
                y = self._new(nd["y"], x.shape, dt)
                self.calls.append((lib.onnx_abs_lp, [B._ptr(x), x.numel(), B._ptr(y), code, None]))
            elif op == "reducesum":
                x = self.t[nd["x"]]
                axes = [] if nd["axes"] is None else list(nd["axes"])
                y = self._new(nd["y"], B.onnx_reduce_infer(x.shape, axes, nd["keepdims"]), dt)
                args = [B._ptr(x), B.dims(x.shape), x.dim(), B.dims(axes), len(axes), int(nd["keepdims"]), B._ptr(y),
                        B.dims(y.shape), y.dim(), code, None]
                self.calls.append((lib.onnx_reducesum_lp, args))
            elif op == "softmax":
                x = self.t[nd["x"]]
                y = self._new(nd["y"], x.shape, dt)
                self.calls.append((lib.onnx_softmax_lp, [B._ptr(x), B.dims(x.shape), x.dim(), int(nd["axis"]), B._ptr(y), code, None]))
            else:                                  # matmul
                a, b = self.t[nd["a"]], self.t[nd["b"]]
                yd = B.onnx_matmul_infer(a.shape, b.shape)
                y = self._new(nd["y"], yd, ydt)
                args = [B._ptr(a), B.dims(a.shape), a.dim(), B._ptr(b), B.dims(b.shape), b.dim(), B._ptr(y),
                        B.dims(y.shape), y.dim(), code, ycode, None]
                self.calls.append((lib.onnx_matmul_lp, args))
        self.output = self.t[model["output"]]

    def _build_chain(self, keep):
        """The model as arguments of one onnx_chain call, or None when it is not a linear chain
        of operators that call takes or the library finds it too large."""
        g = [nd for nd in self.model["graph"]]
        if not g or len(self.model["inputs"]) != 1:
            return None
        cur = next(iter(self.model["inputs"]))
        if self.t[cur].dim() != 4:
            return None
        ops, outs = [], []
        for i, nd in enumerate(g):
            op = nd["op"]
            if op == "reshape":
                x = self.t[nd["x"]]
                nxt = g[i + 1] if i + 1 < len(g) else None
                if nd["x"] != cur or nxt is None or nxt["op"] != "gemm" or tuple(nd["shape"]) != (x.shape[0], x.numel() // max(x.shape[0], 1)):
                    return None
                cur = nd["y"]
                continue
            if op == "conv":
                if nd["x"] != cur or nd["group"] != 1 or nd["residual"]:
                    return None
                ops.append(dict(op="conv", W=self.t[nd["w"]], B=self.t[nd["b"]] if nd["b"] else None, pads=nd["pads"],
                                strides=nd["strides"], dilations=nd["dilations"], act=B.ACT_RELU if nd["relu"] else B.ACT_NONE))
            elif op == "maxpool":
                if nd["x"] != cur:
                    return None
                ops.append(dict(op="maxpool", kernel=nd["kernel"], pads=nd["pads"], strides=nd["strides"],
                                dilations=nd["dilations"], ceil_mode=nd["ceil_mode"]))
            elif op == "avgpool":
                if nd["x"] != cur:
                    return None
                ops.append(dict(op="avgpool", kernel=nd["kernel"], pads=nd["pads"], strides=nd["strides"],
                                ceil_mode=nd["ceil_mode"], count_include_pad=nd["count_include_pad"]))
            elif op == "gemm":
                a, w = self.t[nd["a"]], self.t[nd["b"]]
                c = self.t[nd["c"]] if nd["c"] else None
                n = w.shape[0] if nd["transB"] else w.shape[1]
                if nd["a"] != cur or nd["transA"] or (a.dim() == 4 and a.shape[2] * a.shape[3] != 1):
                    return None
                if c is not None and tuple(c.shape) not in ((n,), (1, n)):
                    return None
                ops.append(dict(op="gemm", W=w, B=c, transB=nd["transB"], alpha=nd["alpha"], beta=nd["beta"],
                                act=B.ACT_RELU if nd["relu"] else B.ACT_NONE))
            else:
                return None
            outs.append(self.t[nd["y"]])
            cur = nd["y"]
        if cur != self.model["output"] or not ops or len(ops) > B.CHAIN_MAX_OPS:
            return None
        x = self.t[next(iter(self.model["inputs"]))]
        arr, results = B.onnx_chain_args(x, ops, keep=keep, outs=outs)
        args = [arr, len(ops), B._ptr(x), B.dims(x.shape), None]
        # the library validates the sizes against what fits on chip; one untimed call finds out
        args[-1] = B._stream(None)
        st = B.raw().onnx_chain(*args)
        if st == B.ONNX_ERR_UNSUPPORTED:
            return None
        if st != B.ONNX_OK:
            raise B.OnnxHipError(st, B.onnx_last_error())
        self._chain_keepalive = (ops, results)
        return (B.raw().onnx_chain, args)

    def _new(self, name, shape, dtype=torch.float32):
        y = torch.empty(tuple(int(s) for s in shape), dtype=dtype, device=self.device)
        self.t[name] = y
        return y

    def set_input(self, name, array):
        self.t[name].copy_(torch.from_numpy(array))        # rounds to the tensor's type (nearest even)

    def capture(self):
        """Record the whole chain into a HIP graph (through torch's stream capture) so that a
        forward pass is one graph launch instead of one host call per node; worthwhile when
        the kernels are so short that launching them is the bottleneck (batch 1)."""
        self.run()
        torch.cuda.synchronize()
        self._graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(self._graph):
            self.run()
        return self

    def replay(self):
        self._graph.replay()
        return self.output

    def run(self, stream=None):
        # The library's workspace is one process-wide setting: point it at this runner's buffer
        # (or clear it) before enqueuing, so that runners never inherit each other's scratch.
        B.onnx_set_workspace(self.workspace)
        sp = B._stream(stream)
        for fn, args in ([self.chain] if self.chain else self.calls):
            args[-1] = sp
            st = fn(*args)
            if st != B.ONNX_OK:
                raise B.OnnxHipError(st, B.onnx_last_error())
        return self.output
