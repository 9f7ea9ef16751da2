"""Tiny model runner: chains library calls for a workload graph.

The analogue of the single entry function a compiled model exports in the paper (Section 3):
the graph's constant inputs are uploaded once, every activation buffer is allocated once, and
``run()`` enqueues one library call per node on one stream with no host synchronisation in
between.  Reshape is a view of dense row-major data and costs nothing.  All arithmetic
happens inside the library's kernels; this module only prepares argument lists.
"""

import torch

from . import binding as B


class GraphRunner:
    def __init__(self, model, device="cuda:0", workspace_bytes=64 << 20):
        self.device = torch.device(device)
        self.model = model
        for nd in model["graph"]:                  # refuse before anything is allocated or registered
            if nd["op"] in ("batchnorm", "identity", "reducel1"):
                raise NotImplementedError(
                    "node %r (%s) has no kernel of its own: run paper_2008_08272_amd.passes.optimize on the "
                    "graph first; it folds, removes or decomposes such nodes" % (nd["y"], nd["op"]))
        # scratch the library may use to split the K range of products with few output tiles
        self.workspace = None
        if workspace_bytes:
            self.workspace = torch.empty(workspace_bytes, dtype=torch.uint8, device=self.device)
            B.onnx_set_workspace(self.workspace)
        self.t = {}
        for k, v in list(model["inputs"].items()) + list(model["weights"].items()):
            self.t[k] = torch.from_numpy(v).to(self.device).contiguous()
        self.calls = []
        self.io = []                 # per call: (names of the tensors it reads, name of the tensor it writes)
        self._alias = {}             # a Reshape result is a view: dependencies go to the tensor behind it
        self._keepalive = []
        lib = B.raw()
        for nd in model["graph"]:
            op = nd["op"]
            ncalls = len(self.calls)
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
            reads = [self._alias.get(nd[f], nd[f]) for f in ("x", "w", "b", "residual", "a", "c") if nd.get(f)]
            if op == "reshape":
                self._alias[nd["y"]] = self._alias.get(nd["x"], nd["x"])
            elif len(self.calls) > ncalls:
                self.io.append((reads, nd["y"]))
        self.output = self.t[model["output"]]
        self._side = None

    def _new(self, name, shape):
        y = torch.empty(tuple(int(s) for s in shape), dtype=torch.float32, device=self.device)
        self.t[name] = y
        return y

    def set_input(self, name, array):
        self.t[name].copy_(torch.from_numpy(array))

    def capture(self, overlap=False):
        """Record the whole chain into a HIP graph (through torch's stream capture) so that a
        forward pass is one graph launch instead of one host call per node; worthwhile when
        the kernels are so short that launching them is the bottleneck (batch 1).  With
        ``overlap`` independent branches of the graph are recorded on a second stream, so the
        HIP graph lets them run side by side (see run_overlapped); measured on ResNet-50 this
        only pays from batch 4 on (0.98 vs 1.02 ms), at batch 1 and 2 the cross-stream
        dependencies cost more than the overlap gains (0.79 vs 0.75 ms), hence off by default."""
        runner = self.run_overlapped if overlap else self.run
        runner()
        torch.cuda.synchronize()
        self._graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(self._graph):
            runner()
        return self

    def run_overlapped(self):
        """Like run(), on two streams: a node that does not read the result of the node before it
        (ResNet's projection shortcut next to the block's first two convolutions) goes to a side
        stream and runs while the main stream continues; events carry the true dependencies.
        At small batch each kernel fills only part of the GPU, so the branches overlap.  Each
        stream's calls get their own half of the workspace (the library uses whichever workspace is
        set when a call is made), so concurrent split-K products do not share scratch memory."""
        main = torch.cuda.current_stream()
        if self._side is None:
            self._side = torch.cuda.Stream(device=self.device)
        side = self._side
        halves = None
        if self.workspace is not None:
            half = (self.workspace.numel() // 2) // 256 * 256
            halves = {main: self.workspace[:half], side: self.workspace[half:2 * half]}
        done = {}                    # tensor name -> (stream that produced it, event recorded behind the producer)
        prev_main = None
        pending_side = []
        for (fn, args), (reads, y) in zip(self.calls, self.io):
            on_side = prev_main is not None and prev_main not in reads
            st_ = side if on_side else main
            for name in reads:
                if name in done and done[name][0] is not st_:
                    st_.wait_event(done[name][1])
            if on_side and not any(name in done for name in reads):
                st_.wait_stream(main)            # reads only graph inputs: still has to join the capture
            if halves is not None:
                B.onnx_set_workspace(halves[st_])
            args[-1] = B._stream(st_)
            rc = fn(*args)
            if rc != B.ONNX_OK:
                raise B.OnnxHipError(rc, B.onnx_last_error())
            ev = torch.cuda.Event()
            ev.record(st_)
            done[y] = (st_, ev)
            if on_side:
                pending_side.append(ev)
            else:
                prev_main = y
        for ev in pending_side:                  # join: the main stream ends behind everything
            main.wait_event(ev)
        if self.workspace is not None:
            B.onnx_set_workspace(self.workspace)
        return self.output

    def replay(self):
        self._graph.replay()
        return self.output

    def run(self, stream=None):
        sp = B._stream(stream)
        for fn, args in self.calls:
            args[-1] = sp
            st = fn(*args)
            if st != B.ONNX_OK:
                raise B.OnnxHipError(st, B.onnx_last_error())
        return self.output
