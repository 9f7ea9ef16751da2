"""Graph-level passes: from the graph an exporter writes to the graph the runner executes.

The paper rewrites the operator graph before lowering it (Section 3.4): shape inference,
MatMul followed by Add becomes Gemm (its MulAddToGemmPattern example), identity operators are
removed, and computations on constants are folded.  The same rewrites are done here on the
runner's graph description (a list of node dicts over named tensors), so that what reaches the
GPU is one library call per fused operator:

    infer_shapes          extents of every tensor (the library's own shape-inference entry points)
    decompose_reducel1    ReduceL1(x) -> ReduceSum(Abs(x))
    eliminate_identity    Identity(x) -> x
    propagate_constants   element-wise operators on constants only are evaluated now; Adds that mix
                          constants and activations are normalised so that the constants meet
    fold_batchnorm        Conv with constant filters + BatchNormalization with constant
                          parameters -> Conv with rescaled filters and a bias
    matmul_add_to_gemm    Add(MatMul(A, B), C) -> Gemm(A, B, C)
    fuse_epilogue         Conv/Gemm [+ Add(residual)] [+ Relu] -> one node with the epilogue flags

Every pass takes a model dict and returns a new one; none touches the GPU.  ``optimize`` runs
them all.  A Relu or Add that found no producer to fuse into stays a node of its own and runs
through the library's element-wise kernels; nodes the runner cannot execute (a
BatchNormalization on a non-constant input, a ReduceL1 that was not decomposed, an Identity)
make it raise: there is no slow path.
"""

import numpy as np

from . import binding as B

# tensor-valued fields of each node kind (inputs), used for use counting and renaming
_INPUTS = {
    "conv": ("x", "w", "b", "residual"),
    "gemm": ("a", "b", "c"),
    "matmul": ("a", "b"),
    "maxpool": ("x",),
    "avgpool": ("x",),
    "reshape": ("x",),
    "batchnorm": ("x", "scale", "bias", "mean", "var"),
    "relu": ("x",),
    "add": ("a", "b"),
    "identity": ("x",),
    "leakyrelu": ("x",),
    "abs": ("x",),
    "reducesum": ("x",),
    "reducel1": ("x",),
    "softmax": ("x",),
}


def _clone(model, graph=None, weights=None):
    out = dict(model)
    out["graph"] = [dict(nd) for nd in (model["graph"] if graph is None else graph)]
    out["weights"] = dict(model["weights"] if weights is None else weights)
    return out


def _uses(model):
    """Number of consumers of every tensor name (the graph output counts as one)."""
    n = {}
    for nd in model["graph"]:
        for f in _INPUTS[nd["op"]]:
            t = nd.get(f)
            if t:
                n[t] = n.get(t, 0) + 1
    n[model["output"]] = n.get(model["output"], 0) + 1
    return n


def _producers(model):
    return {nd["y"]: i for i, nd in enumerate(model["graph"])}


def _rename(model, old, new):
    for nd in model["graph"]:
        for f in _INPUTS[nd["op"]]:
            if nd.get(f) == old:
                nd[f] = new
    if model["output"] == old:
        model["output"] = new


def _drop_unused_weights(model):
    used = set()
    for nd in model["graph"]:
        for f in _INPUTS[nd["op"]]:
            if nd.get(f):
                used.add(nd[f])
    model["weights"] = {k: v for k, v in model["weights"].items() if k in used}
    return model


# ----------------------------------------------------------------------------- shape inference

def infer_shapes(model):
    """Extent of every tensor of the graph, by walking it once (Section 3.4: shape inference is a
    pass of its own, run before the operators are lowered).  Conv, pooling and MatMul extents
    come from the library's ``*_infer`` entry points, so the pass and the kernels cannot
    disagree."""
    sh = {k: tuple(v.shape) for k, v in model["inputs"].items()}
    sh.update({k: tuple(v.shape) for k, v in model["weights"].items()})
    for nd in model["graph"]:
        op = nd["op"]
        if op == "conv":
            y = B.onnx_conv_infer(sh[nd["x"]], sh[nd["w"]], nd["pads"], nd["strides"], nd["dilations"], nd["group"])
        elif op == "maxpool":
            y = B.onnx_pool_infer(sh[nd["x"]], nd["kernel"], nd["pads"], nd["strides"], nd["dilations"], nd["ceil_mode"])
        elif op == "avgpool":
            x = sh[nd["x"]]
            y = (x[0], x[1], 1, 1) if nd["kernel"] is None else \
                B.onnx_pool_infer(x, nd["kernel"], nd["pads"], nd["strides"], (1, 1), nd["ceil_mode"])
        elif op == "reshape":
            y = tuple(nd["shape"])
            if int(np.prod(y)) != int(np.prod(sh[nd["x"]])):
                raise ValueError("reshape %s: %r does not hold %r" % (nd["y"], y, sh[nd["x"]]))
        elif op == "gemm":
            a, b = sh[nd["a"]], sh[nd["b"]]
            m, k = (a[1], a[0]) if nd["transA"] else a
            kb, n = (b[1], b[0]) if nd["transB"] else b
            if k != kb:
                raise ValueError("gemm %s: inner extents %d and %d differ" % (nd["y"], k, kb))
            y = (m, n)
        elif op == "matmul":
            y = B.onnx_matmul_infer(sh[nd["a"]], sh[nd["b"]])
        elif op in ("batchnorm", "relu", "identity", "leakyrelu", "abs", "softmax"):
            y = sh[nd["x"]]
        elif op in ("reducesum", "reducel1"):
            y = B.onnx_reduce_infer(sh[nd["x"]], nd["axes"], nd["keepdims"])
        elif op == "add":
            y = B.onnx_broadcast_infer(sh[nd["a"]], sh[nd["b"]])
        else:
            raise ValueError("unknown node op %r" % (op,))
        sh[nd["y"]] = tuple(int(d) for d in y)
    return sh


# ----------------------------------------------------------------------------- rewrites

def decompose_reducel1(model):
    """ReduceL1(x, axes, keepdims) -> ReduceSum(Abs(x), axes, keepdims): the operator
    decomposition the paper gives as its first example of a rewriting pass (Section 3.4), so
    that only ReduceSum and Abs need kernels."""
    out = _clone(model)
    graph = []
    for nd in out["graph"]:
        if nd["op"] == "reducel1":
            tmp = nd["y"] + "_abs"
            graph.append(dict(op="abs", x=nd["x"], y=tmp))
            graph.append(dict(op="reducesum", x=tmp, y=nd["y"], axes=nd["axes"], keepdims=nd["keepdims"]))
        else:
            graph.append(nd)
    out["graph"] = graph
    return out


def eliminate_identity(model):
    out = _clone(model)
    for nd in list(out["graph"]):
        if nd["op"] == "identity":
            out["graph"].remove(nd)
            _rename(out, nd["y"], nd["x"])
    return out


def fold_batchnorm(model):
    """Conv(x, W, b) -> BatchNormalization(scale, bias, mean, var, eps), all parameters constant
    and the convolution's result used by nothing else, becomes Conv(x, W', b') with
        s = scale / sqrt(var + eps),   W'[m] = W[m] * s[m],   b'[m] = (b[m] - mean[m]) * s[m] + bias[m]
    computed in double and rounded to fp32 once (constant folding, Section 3.4)."""
    out = _clone(model)
    w = out["weights"]
    changed = True
    while changed:
        changed = False
        uses, prod = _uses(out), _producers(out)
        for bn in out["graph"]:
            if bn["op"] != "batchnorm" or bn["x"] not in prod:
                continue
            cv = out["graph"][prod[bn["x"]]]
            consts = [bn["scale"], bn["bias"], bn["mean"], bn["var"], cv.get("w")] + ([cv["b"]] if cv.get("b") else [])
            if cv["op"] != "conv" or uses[cv["y"]] != 1 or cv["relu"] or cv["residual"] or \
                    any(c not in w for c in consts):
                continue
            s = w[bn["scale"]].astype(np.float64) / np.sqrt(w[bn["var"]].astype(np.float64) + bn["eps"])
            b0 = w[cv["b"]].astype(np.float64) if cv.get("b") else 0.0
            wn, bname = cv["y"] + "_wfold", cv["y"] + "_bfold"
            w[wn] = (w[cv["w"]].astype(np.float64) * s[:, None, None, None]).astype(np.float32)
            w[bname] = ((b0 - w[bn["mean"]].astype(np.float64)) * s + w[bn["bias"]].astype(np.float64)).astype(np.float32)
            cv["w"], cv["b"], cv["y"] = wn, bname, bn["y"]
            out["graph"].remove(bn)
            changed = True
            break
    return _drop_unused_weights(out)


def _fold_constant_nodes(out):
    """Evaluates Add / Relu / Abs / LeakyRelu / Identity / Reshape nodes whose inputs are all
    constants (fp32, one rounding per operator, as the kernels would) and makes their results
    constants of the graph."""
    w = out["weights"]
    changed = False
    for nd in list(out["graph"]):
        op = nd["op"]
        if op not in ("add", "relu", "abs", "leakyrelu", "identity", "reshape"):
            continue
        ins = [nd[f] for f in _INPUTS[op] if nd.get(f)]
        if not ins or any(t not in w for t in ins) or nd["y"] == out["output"]:
            continue
        if op == "add":
            v = w[nd["a"]] + w[nd["b"]]
        elif op == "relu":
            v = np.where(w[nd["x"]] > 0, w[nd["x"]], np.float32(0))
        elif op == "abs":
            v = np.abs(w[nd["x"]])
        elif op == "leakyrelu":
            v = np.where(w[nd["x"]] >= 0, w[nd["x"]], np.float32(nd["alpha"]) * w[nd["x"]])
        elif op == "reshape":
            v = np.reshape(w[nd["x"]], nd["shape"])
        else:
            v = w[nd["x"]]
        w[nd["y"]] = np.ascontiguousarray(v, dtype=np.float32)
        out["graph"].remove(nd)
        changed = True
    return changed


def propagate_constants(model):
    """Constant propagation (Section 3.4).  An operator all of whose inputs are constants is
    evaluated here and removed (element-wise operators and Reshape; BatchNormalization on a
    convolution is fold_batchnorm's business).  Adds that mix constants c and activations x, y
    are normalised with the paper's rules, which move the constants outwards until they meet:
        c + x               ->  x + c
        (x + c1) + c2       ->  x + (c1 + c2)
        (x + c) + y         ->  (x + y) + c
        x + (y + c)         ->  (x + y) + c
        (x + c1) + (y + c2) ->  (x + y) + (c1 + c2)
    An inner Add is only taken apart when nothing else reads its result.  The sum of two
    constants is formed in fp32 like any Add, so the rewritten graph differs from the original
    by the rounding of a reassociated fp32 sum, not more."""
    out = _clone(model)
    w = out["weights"]
    counter = [0]

    def fresh(stem):
        counter[0] += 1
        return "%s_cp%d" % (stem, counter[0])

    changed = True
    while changed:
        changed = _fold_constant_nodes(out)
        uses, prod = _uses(out), _producers(out)

        def const_add(name):
            """(x, c) when `name` is the single-use result of Add(x, c) with c constant, x not."""
            if name not in prod or uses.get(name, 0) != 1:
                return None
            nd = out["graph"][prod[name]]
            if nd["op"] == "add" and nd["b"] in w and nd["a"] not in w:
                return nd
            return None

        for nd in out["graph"]:
            if nd["op"] != "add":
                continue
            a, b = nd["a"], nd["b"]
            if a in w and b not in w:                                  # c + x -> x + c
                nd["a"], nd["b"] = b, a
                changed = True
                break
            if a in w:
                continue                                               # both constant: folded above
            ia, ib = const_add(a), (None if b in w else const_add(b))
            if b in w and ia is not None:                              # (x + c1) + c2 -> x + (c1 + c2)
                c = fresh("c")
                w[c] = np.ascontiguousarray(w[ia["b"]] + w[b], dtype=np.float32)
                nd["a"], nd["b"] = ia["a"], c
                out["graph"].remove(ia)
                changed = True
                break
            if b in w:
                continue
            if ia is not None and ib is not None:                      # (x + c1) + (y + c2) -> (x + y) + (c1 + c2)
                c, t = fresh("c"), fresh(nd["y"])
                w[c] = np.ascontiguousarray(w[ia["b"]] + w[ib["b"]], dtype=np.float32)
                i = out["graph"].index(nd)
                out["graph"][i:i + 1] = [dict(op="add", a=ia["a"], b=ib["a"], y=t), dict(op="add", a=t, b=c, y=nd["y"])]
                out["graph"].remove(ia)
                out["graph"].remove(ib)
                changed = True
                break
            inner, other = (ia, b) if ia is not None else (ib, a)
            if inner is not None:                                      # (x + c) + y  /  x + (y + c) -> (x + y) + c
                t = fresh(nd["y"])
                first, second = (inner["a"], other) if inner is ia else (other, inner["a"])
                i = out["graph"].index(nd)
                out["graph"][i:i + 1] = [dict(op="add", a=first, b=second, y=t), dict(op="add", a=t, b=inner["b"], y=nd["y"])]
                out["graph"].remove(inner)
                changed = True
                break
    return _drop_unused_weights(out)


def matmul_add_to_gemm(model):
    """Add(MatMul(A, B), C) with 2-D A and B, the product used only by the Add, and C
    broadcastable to the product's shape, becomes Gemm(A, B, C) with alpha = beta = 1 (the
    paper's MulAddToGemmPattern, Section 3.4)."""
    out = _clone(model)
    changed = True
    while changed:
        changed = False
        sh, uses, prod = infer_shapes(out), _uses(out), _producers(out)
        for ad in out["graph"]:
            if ad["op"] != "add":
                continue
            for mm_name, c_name in ((ad["a"], ad["b"]), (ad["b"], ad["a"])):
                if mm_name not in prod:
                    continue
                mm = out["graph"][prod[mm_name]]
                if mm["op"] != "matmul" or uses[mm_name] != 1 or len(sh[mm["a"]]) != 2 or len(sh[mm["b"]]) != 2:
                    continue
                m, n = sh[mm_name]
                if sh[c_name] not in ((), (1,), (n,), (1, n), (m, 1), (m, n), (1, 1)):
                    continue
                if c_name in prod and prod[c_name] > prod[mm_name]:
                    continue                       # C is computed after the product: leave the pair alone
                i = out["graph"].index(mm)
                out["graph"][i] = dict(op="gemm", a=mm["a"], b=mm["b"], c=c_name, y=ad["y"], alpha=1.0,
                                       beta=1.0, transA=0, transB=0, relu=False)
                out["graph"].remove(ad)
                changed = True
                break
            if changed:
                break
    return out


def fuse_epilogue(model):
    """Folds Add(conv result, other) and Relu(conv or gemm result) into the producing node's
    epilogue (the kernels apply  relu?(acc + bias + residual)  before the store), when the
    intermediate result has no other consumer.  For an Add of two convolution results the later
    node takes the earlier one's result as its residual."""
    out = _clone(model)
    changed = True
    while changed:
        changed = False
        sh, uses, prod = infer_shapes(out), _uses(out), _producers(out)
        for nd in out["graph"]:
            if nd["op"] == "add":
                cands = [(prod[t], t, o) for t, o in ((nd["a"], nd["b"]), (nd["b"], nd["a"])) if t in prod]
                for pi, t, other in sorted(cands, reverse=True):
                    cv = out["graph"][pi]
                    if cv["op"] != "conv" or uses[t] != 1 or cv["relu"] or cv["residual"] or sh[other] != sh[t]:
                        continue
                    if other in prod and prod[other] > pi:
                        continue                   # the other operand does not exist yet when cv runs
                    cv["residual"], cv["y"] = other, nd["y"]
                    out["graph"].remove(nd)
                    changed = True
                    break
            elif nd["op"] == "relu" and nd["x"] in prod:
                pr = out["graph"][prod[nd["x"]]]
                if pr["op"] in ("conv", "gemm") and uses[nd["x"]] == 1 and not pr["relu"]:
                    pr["relu"], pr["y"] = True, nd["y"]
                    out["graph"].remove(nd)
                    changed = True
            if changed:
                break
    return out


def optimize(model):
    """All passes, in the order that lets each see the patterns the previous one exposed."""
    m = decompose_reducel1(model)
    m = eliminate_identity(m)
    m = propagate_constants(m)
    m = fold_batchnorm(m)
    m = matmul_add_to_gemm(m)
    m = fuse_epilogue(m)
    infer_shapes(m)                                  # the rewritten graph must still be well-formed
    return _drop_unused_weights(m)
