"""Seeded synthetic inputs and graph descriptions for the five workloads.

This module is shared by the CPU oracle's tests and by the GPU library's tests,
benchmark and runner.  It draws random tensors and lists the operator nodes of
each model; it performs none of the operators' arithmetic.  (The one numerical
step here is the offline folding of BatchNorm statistics into convolution weights
and biases, which is part of preparing ResNet-50's constant inputs: both sides
receive the same folded fp32 arrays.)

The models stand in for the ONNX Model Zoo MNIST and ResNet50 networks used in
the paper's experiments (Section 4.2): same operator mix, tensor shapes and
fp32 element type; all values random.

A graph is a list of node dicts executed in order.  Tensor names refer to
entries of ``inputs`` / ``weights`` or to an earlier node's ``y``:

  conv     x w b pads strides dilations group residual relu y
  maxpool  x kernel pads strides dilations ceil_mode y
  avgpool  x kernel(None = global) pads strides ceil_mode count_include_pad y
  reshape  x shape y                       (a view of dense row-major data)
  gemm     a b c alpha beta transA transB relu y
  matmul   a b y

Graphs "as an exporter writes them" (the inputs of the graph-level passes) also use

  batchnorm x scale bias mean var eps y      relu x y        add a b y       identity x y
  leakyrelu x alpha y     abs x y     reducesum / reducel1 x axes keepdims y     softmax x axis y
"""
import numpy as np

SEED_BASE = 20080827


def _rng(seed, stream):
    return np.random.default_rng([int(seed), int(stream)])


def _uniform(rng, shape, lo=-1.0, hi=1.0):
    return rng.uniform(lo, hi, size=shape).astype(np.float32)


def _normal(rng, shape, std):
    return (rng.standard_normal(size=shape) * std).astype(np.float32)


def conv_node(x, w, b, y, pads=(0, 0, 0, 0), strides=(1, 1), dilations=(1, 1), group=1,
              residual=None, relu=False):
    return dict(op="conv", x=x, w=w, b=b, y=y, pads=tuple(pads), strides=tuple(strides),
                dilations=tuple(dilations), group=group, residual=residual, relu=relu)


def maxpool_node(x, y, kernel, pads=(0, 0, 0, 0), strides=(1, 1), dilations=(1, 1), ceil_mode=0):
    return dict(op="maxpool", x=x, y=y, kernel=tuple(kernel), pads=tuple(pads),
                strides=tuple(strides), dilations=tuple(dilations), ceil_mode=ceil_mode)


def avgpool_node(x, y, kernel=None, pads=(0, 0, 0, 0), strides=(1, 1), ceil_mode=0,
                 count_include_pad=0):
    return dict(op="avgpool", x=x, y=y, kernel=None if kernel is None else tuple(kernel),
                pads=tuple(pads), strides=tuple(strides), ceil_mode=ceil_mode,
                count_include_pad=count_include_pad)


def gemm_node(a, b, c, y, alpha=1.0, beta=1.0, transA=0, transB=0, relu=False):
    return dict(op="gemm", a=a, b=b, c=c, y=y, alpha=alpha, beta=beta, transA=transA,
                transB=transB, relu=relu)


def reshape_node(x, y, shape):
    return dict(op="reshape", x=x, y=y, shape=tuple(shape))


# Nodes that only occur in graphs as an exporter would write them, before any graph-level pass
# (Section 3.4 of the paper: operators are fused and constants folded by rewriting the graph).
def batchnorm_node(x, scale, bias, mean, var, y, eps):
    return dict(op="batchnorm", x=x, scale=scale, bias=bias, mean=mean, var=var, y=y, eps=float(eps))


def relu_node(x, y):
    return dict(op="relu", x=x, y=y)


def add_node(a, b, y):
    return dict(op="add", a=a, b=b, y=y)


def identity_node(x, y):
    return dict(op="identity", x=x, y=y)


def matmul_node(a, b, y):
    return dict(op="matmul", a=a, b=b, y=y)


def leakyrelu_node(x, y, alpha=0.01):
    return dict(op="leakyrelu", x=x, y=y, alpha=float(alpha))


def abs_node(x, y):
    return dict(op="abs", x=x, y=y)


def reduce_node(kind, x, y, axes=None, keepdims=1):
    """kind: "reducesum" or "reducel1" (the latter exists only before the decomposition pass)."""
    return dict(op=kind, x=x, y=y, axes=None if axes is None else tuple(int(a) for a in axes),
                keepdims=int(keepdims))


def softmax_node(x, y, axis=-1):
    return dict(op="softmax", x=x, y=y, axis=int(axis))


# --------------------------------------------------------------------------- config 1

def small_cnn(seed=SEED_BASE + 1):
    """MNIST-shaped CNN, batch 1: conv5x5(8)+Relu, maxpool 2/2, conv5x5(16)+Relu,
    maxpool 3/3, reshape 1x256, Gemm 256x10 + bias.  X ~ U[0,1), weights N(0, 0.1^2),
    biases N(0, 0.01^2), all from one generator in the order listed."""
    r = _rng(seed, 0)
    inputs = {"x": _uniform(r, (1, 1, 28, 28), 0.0, 1.0)}
    weights = {}
    weights["w1"] = _normal(r, (8, 1, 5, 5), 0.1)
    weights["b1"] = _normal(r, (8,), 0.01)
    weights["w2"] = _normal(r, (16, 8, 5, 5), 0.1)
    weights["b2"] = _normal(r, (16,), 0.01)
    weights["wg"] = _normal(r, (256, 10), 0.1)
    weights["bg"] = _normal(r, (1, 10), 0.01)
    graph = [
        conv_node("x", "w1", "b1", "c1", pads=(2, 2, 2, 2), relu=True),
        maxpool_node("c1", "p1", (2, 2), strides=(2, 2)),
        conv_node("p1", "w2", "b2", "c2", pads=(2, 2, 2, 2), relu=True),
        maxpool_node("c2", "p2", (3, 3), strides=(3, 3)),
        reshape_node("p2", "flat", (1, 256)),
        gemm_node("flat", "wg", "bg", "logits"),
    ]
    return dict(name="small_cnn", inputs=inputs, weights=weights, graph=graph, output="logits")


def small_cnn_unfused(seed=SEED_BASE + 1):
    """The same network and tensors as ``small_cnn`` written operator by operator: Relu as
    nodes of their own, the classifier as MatMul followed by Add (the pair the paper's
    MatMul+Add -> Gemm rewrite targets, Section 3.4), and an Identity on the input."""
    m = small_cnn(seed)
    graph = [
        identity_node("x", "x_id"),
        conv_node("x_id", "w1", "b1", "c1_lin", pads=(2, 2, 2, 2)),
        relu_node("c1_lin", "c1"),
        maxpool_node("c1", "p1", (2, 2), strides=(2, 2)),
        conv_node("p1", "w2", "b2", "c2_lin", pads=(2, 2, 2, 2)),
        relu_node("c2_lin", "c2"),
        maxpool_node("c2", "p2", (3, 3), strides=(3, 3)),
        reshape_node("p2", "flat", (1, 256)),
        matmul_node("flat", "wg", "mm"),
        add_node("mm", "bg", "logits"),
    ]
    return dict(name="small_cnn_unfused", inputs=m["inputs"], weights=m["weights"], graph=graph,
                output="logits")


def classifier_head(batch=32, classes=1000, features=2048, seed=SEED_BASE + 6):
    """A classifier tail written operator by operator, exercising the element-wise, reduction
    and softmax operators: features -> LeakyRelu -> MatMul + Add (-> Gemm) -> Softmax, plus the L1
    norm of the logits per image (ReduceL1, which the decomposition pass turns into Abs +
    ReduceSum) and the column sums of the probabilities."""
    r = _rng(seed, 0)
    inputs = {"feat": _normal(r, (batch, features), 1.0)}
    weights = {"w": _normal(r, (features, classes), np.sqrt(1.0 / features)),
               "b": _normal(r, (classes,), 0.1)}
    graph = [
        leakyrelu_node("feat", "act", 0.1),
        matmul_node("act", "w", "mm"),
        add_node("mm", "b", "logits"),
        softmax_node("logits", "prob", axis=1),
        reduce_node("reducel1", "logits", "l1", axes=(1,), keepdims=0),
        reduce_node("reducesum", "prob", "colsum", axes=(0,), keepdims=1),
    ]
    return dict(name="classifier_head", inputs=inputs, weights=weights, graph=graph, output="prob")


def constant_adds(batch=4, channels=16, hw=12, seed=SEED_BASE + 8):
    """A graph with chained Adds of constants around two activations, every shape of the paper's
    Add normalisation rules (Section 3.4, constant propagation) once, plus an Add and a Relu of
    constants only:  x, y = Relu(x)  ->  c1 + x,  (x + c1) + c2,  (x + c) + y,  x + (y + c),
    (x + c1) + (y + c2), with per-channel, scalar and full-tensor constants."""
    r = _rng(seed, 0)
    inputs = {"x": _normal(r, (batch, channels, hw, hw), 1.0)}
    weights = {"c1": _normal(r, (1, channels, 1, 1), 1.0), "c2": _normal(r, (1, channels, 1, 1), 1.0),
               "c3": np.asarray(_normal(r, (1,), 1.0)[0], dtype=np.float32), "c4": _normal(r, (channels, hw, hw), 1.0),
               "c5": _normal(r, (1, channels, 1, 1), 1.0), "c6": _normal(r, (hw,), 1.0)}
    graph = [
        relu_node("x", "y"),
        add_node("c1", "x", "t1"),            # c + x
        add_node("t1", "c2", "t2"),           # (x + c1) + c2
        add_node("t2", "y", "t3"),            # (x + c) + y
        add_node("c5", "c6", "k1"),           # constants only
        relu_node("k1", "k2"),                # constants only
        add_node("y", "k2", "t4"),            # y + c
        add_node("t3", "t4", "t5"),           # (u + c) + (y + c')
        add_node("x", "c3", "t6"),            # x + c
        add_node("t5", "t6", "t7"),           # u + (x + c)
        add_node("t7", "c4", "out"),
    ]
    return dict(name="constant_adds", inputs=inputs, weights=weights, graph=graph, output="out")


# --------------------------------------------------------------------------- config 2

def gemm_case(n, seed=SEED_BASE + 2, m=None, k=None):
    """One case of the Gemm sweep: A[M,K], B[N,K] (transB=1), C[1,N], all U[-1,1).
    The stream index is the problem size so each size has its own tensors."""
    m = n if m is None else m
    k = n if k is None else k
    r = _rng(seed, n)
    return dict(A=_uniform(r, (m, k)), B=_uniform(r, (n, k)), C=_uniform(r, (1, n)),
                alpha=1.0, beta=1.0, transA=0, transB=1)


GEMM_SWEEP_SIZES = (1024, 2048, 4096)


def to_bf16_bits(x):
    """fp32 array -> bfloat16 storage (uint16: the upper half of the binary32 pattern), rounded to
    nearest even.  Input preparation only."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)


def from_bf16_bits(b):
    """bfloat16 storage -> the fp32 values it denotes (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def gemm_case_16bit(n, kind, seed=SEED_BASE + 7, m=None, k=None):
    """A [m,k], B [n,k] (used with transB=1) drawn U[-1,1) and rounded to ``kind`` ("f16" or "bf16"),
    C [1,n] fp32.  Returns the 16-bit storage (uint16 bit patterns) and the fp32 values they
    denote, which is what a reference has to be computed from."""
    m = n if m is None else m
    k = n if k is None else k
    r = _rng(seed, n)
    a, b, c = _uniform(r, (m, k)), _uniform(r, (n, k)), _uniform(r, (1, n))
    if kind == "bf16":
        ab, bb = to_bf16_bits(a), to_bf16_bits(b)
        av, bv = from_bf16_bits(ab), from_bf16_bits(bb)
    elif kind == "f16":
        ah, bh = a.astype(np.float16), b.astype(np.float16)
        ab, bb = ah.view(np.uint16), bh.view(np.uint16)
        av, bv = ah.astype(np.float32), bh.astype(np.float32)
    else:
        raise ValueError(kind)
    return dict(A_bits=ab, B_bits=bb, A=av, B=bv, C=c, kind=kind)


# --------------------------------------------------------------------------- configs 3, 4

RESNET50_STAGES = ((64, 3, 1), (128, 4, 2), (256, 6, 2), (512, 3, 2))   # width, blocks, stride
BN_EPS = 1e-5


def _folded_conv(r, cout, cin, k):
    """He-normal conv weight (std = sqrt(2/fan_in), zero conv bias) followed by a BatchNorm with
    gamma ~ U[0.8,1.2], var ~ U[0.8,1.2], mean ~ N(0,0.1^2), beta ~ N(0,0.1^2), eps 1e-5,
    folded in double: s = gamma/sqrt(var+eps); W' = W*s; b' = beta - mean*s."""
    fan_in = cin * k * k
    w = r.standard_normal(size=(cout, cin, k, k)) * np.sqrt(2.0 / fan_in)
    w = w.astype(np.float32).astype(np.float64)
    gamma = r.uniform(0.8, 1.2, size=cout)
    var = r.uniform(0.8, 1.2, size=cout)
    mean = r.standard_normal(size=cout) * 0.1
    beta = r.standard_normal(size=cout) * 0.1
    s = gamma / np.sqrt(var + BN_EPS)
    wf = (w * s[:, None, None, None]).astype(np.float32)
    bf = (beta - mean * s).astype(np.float32)
    raw = dict(w=w.astype(np.float32), gamma=gamma, var=var, mean=mean, beta=beta)
    return wf, bf, raw


def resnet50(batch=1, seed=None, keep_raw=False, image=224):
    """ResNet-50 v1 inference graph with BatchNorm folded.  Stem 7x7/2 pad 3 + Relu,
    maxpool 3x3/2 pad 1; bottlenecks [3,4,6,3] (1x1 -> 3x3 -> 1x1, expansion 4) with the stride
    on the 3x3 conv and on the 1x1 projection of each stage's first block; Relu after conv a,
    conv b and after the residual add; global average pool; Gemm 2048 -> 1000 (W stored
    [1000,2048], transB=1).  The weights always come from the batch-1 seed so both batch sizes
    share them; the image batch comes from ``seed``."""
    wseed = SEED_BASE + 3
    if seed is None:
        seed = SEED_BASE + (3 if batch == 1 else 4)
    rx = _rng(seed, 0)
    rw = _rng(wseed, 1)
    inputs = {"x": _normal(rx, (batch, 3, image, image), 1.0)}
    weights, graph, raws = {}, [], {}

    def add_conv(name, x, cout, cin, k, stride, pad, relu, residual=None):
        wf, bf, raw = _folded_conv(rw, cout, cin, k)
        weights[name + "_w"], weights[name + "_b"] = wf, bf
        if keep_raw:
            raws[name] = raw
        graph.append(conv_node(x, name + "_w", name + "_b", name, pads=(pad,) * 4,
                               strides=(stride, stride), residual=residual, relu=relu))
        return name

    cur = add_conv("stem", "x", 64, 3, 7, 2, 3, True)
    graph.append(maxpool_node(cur, "pool0", (3, 3), pads=(1, 1, 1, 1), strides=(2, 2)))
    cur, cin = "pool0", 64
    for si, (width, blocks, stride) in enumerate(RESNET50_STAGES, start=1):
        for bi in range(blocks):
            p = "s%db%d" % (si, bi)
            s = stride if bi == 0 else 1
            a = add_conv(p + "a", cur, width, cin, 1, 1, 0, True)
            b = add_conv(p + "b", a, width, width, 3, s, 1, True)
            if bi == 0:
                short = add_conv(p + "p", cur, width * 4, cin, 1, s, 0, False)
            else:
                short = cur
            cur = add_conv(p + "c", b, width * 4, width, 1, 1, 0, True, residual=short)
            cin = width * 4
    graph.append(avgpool_node(cur, "gap", None))
    graph.append(reshape_node("gap", "feat", (batch, 2048)))
    weights["fc_w"] = _normal(rw, (1000, 2048), np.sqrt(2.0 / 2048))
    weights["fc_b"] = _normal(rw, (1, 1000), 0.01)
    graph.append(gemm_node("feat", "fc_w", "fc_b", "logits", transB=1))
    out = dict(name="resnet50_b%d" % batch, inputs=inputs, weights=weights, graph=graph,
               output="logits")
    if keep_raw:
        out["raw"] = raws
    return out


def resnet50_unfused(batch=1, seed=None, image=224):
    """The network of ``resnet50`` as an exporter writes it: every convolution without bias,
    followed by a BatchNormalization node (fp32 scale, bias, mean, var; eps 1e-5), Relu and the
    residual Add as nodes of their own.  Same random draws as ``resnet50``; the BatchNorm
    parameters are stored in fp32, as a model file would hold them."""
    m = resnet50(batch, seed, keep_raw=True, image=image)
    weights, graph = {}, []
    for nd in m["graph"]:
        if nd["op"] != "conv":
            graph.append(dict(nd))
            for k in ("b", "c"):
                if nd["op"] == "gemm" and nd.get(k):
                    weights[nd[k]] = m["weights"][nd[k]]
            continue
        name, raw = nd["y"], m["raw"][nd["y"]]
        weights[name + "_w"] = raw["w"]
        for k in ("gamma", "beta", "mean", "var"):
            weights[name + "_" + k] = np.asarray(raw[k], dtype=np.float32)
        graph.append(conv_node(nd["x"], name + "_w", None, name + "_conv", pads=nd["pads"],
                               strides=nd["strides"], dilations=nd["dilations"], group=nd["group"]))
        bn_out = name if not (nd["residual"] or nd["relu"]) else name + "_bn"
        graph.append(batchnorm_node(name + "_conv", name + "_gamma", name + "_beta", name + "_mean",
                                    name + "_var", bn_out, BN_EPS))
        cur = bn_out
        if nd["residual"]:
            nxt = name if not nd["relu"] else name + "_sum"
            graph.append(add_node(cur, nd["residual"], nxt))
            cur = nxt
        if nd["relu"]:
            graph.append(relu_node(cur, name))
    return dict(name="resnet50_unfused_b%d" % batch, inputs=m["inputs"], weights=weights, graph=graph,
                output=m["output"])


# --------------------------------------------------------------------------- config 5

def attr_sweep_case(which, seed=SEED_BASE + 5, batch=None):
    """Attribute-coverage cases, U[-1,1) data.  ``batch`` shrinks the leading dimension for tests
    that run the oracle on a few images only (the tensors drawn are then a prefix-independent
    draw of their own, not a slice of the full case)."""
    cases = {
        "depthwise": dict(x=(8, 256, 56, 56), w=(256, 1, 3, 3), pads=(1, 1, 1, 1), strides=(1, 1),
                          dilations=(1, 1), group=256),
        "dilated": dict(x=(8, 512, 28, 28), w=(512, 512, 3, 3), pads=(2, 2, 2, 2), strides=(1, 1),
                        dilations=(2, 2), group=1),
        "pointwise": dict(x=(32, 1024, 14, 14), w=(256, 1024, 1, 1), pads=(0, 0, 0, 0),
                          strides=(1, 1), dilations=(1, 1), group=1),
    }
    mm = {"matmul_heads": ((8, 12, 512, 64), (8, 12, 64, 512)),
          "matmul_proj": ((8, 512, 768), (768, 3072))}
    stream = sorted(list(cases) + list(mm)).index(which)
    r = _rng(seed, stream)
    if which in cases:
        c = dict(cases[which])
        xs = list(c.pop("x"))
        if batch is not None:
            xs[0] = batch
        ws = c.pop("w")
        c.update(X=_uniform(r, xs), W=_uniform(r, ws), B=_uniform(r, (ws[0],)))
        return c
    a, b = mm[which]
    if batch is not None:
        a = (batch,) + a[1:]
        if len(b) == len(a):
            b = (batch,) + b[1:]
    return dict(A=_uniform(r, a), B=_uniform(r, b))


ATTR_SWEEP_CONV = ("depthwise", "dilated", "pointwise")
ATTR_SWEEP_MATMUL = ("matmul_heads", "matmul_proj")


# --------------------------------------------------------------------------- bookkeeping

def window_out(n, k, pb, pe, s, d=1):
    return (n + pb + pe - ((k - 1) * d + 1)) // s + 1


def graph_stats(model):
    """Parameter count and nominal MACs (padded taps counted) of a graph, by shape walking."""
    shapes = {k: v.shape for k, v in model["inputs"].items()}
    shapes.update({k: v.shape for k, v in model["weights"].items()})
    params = sum(int(np.prod(v.shape)) for v in model["weights"].values())
    macs, per_node = 0, []
    for nd in model["graph"]:
        op = nd["op"]
        if op == "conv":
            n, c, h, w = shapes[nd["x"]]
            m, cg, kh, kw = shapes[nd["w"]]
            oh = window_out(h, kh, nd["pads"][0], nd["pads"][2], nd["strides"][0], nd["dilations"][0])
            ow = window_out(w, kw, nd["pads"][1], nd["pads"][3], nd["strides"][1], nd["dilations"][1])
            shapes[nd["y"]] = (n, m, oh, ow)
            mac = n * m * oh * ow * cg * kh * kw
        elif op in ("maxpool", "avgpool"):
            n, c, h, w = shapes[nd["x"]]
            if nd["kernel"] is None:
                oh = ow = 1
            else:
                d = nd.get("dilations", (1, 1))
                oh = window_out(h, nd["kernel"][0], nd["pads"][0], nd["pads"][2], nd["strides"][0], d[0])
                ow = window_out(w, nd["kernel"][1], nd["pads"][1], nd["pads"][3], nd["strides"][1], d[1])
            shapes[nd["y"]] = (n, c, oh, ow)
            mac = 0
        elif op == "reshape":
            shapes[nd["y"]] = nd["shape"]
            mac = 0
        elif op == "gemm":
            a, b = shapes[nd["a"]], shapes[nd["b"]]
            mm, kk = (a[1], a[0]) if nd["transA"] else a
            nn = b[0] if nd["transB"] else b[1]
            shapes[nd["y"]] = (mm, nn)
            mac = mm * nn * kk
        else:
            raise ValueError(op)
        macs += mac
        # compulsory bytes of the node: every operand read once, the result written once
        operands = [nd.get(k) for k in ("x", "w", "b", "residual", "a", "c")]
        if op == "gemm":
            operands = [nd["a"], nd["b"], nd.get("c")]
        nbytes = 0 if op == "reshape" else 4 * (sum(int(np.prod(shapes[k])) for k in operands if k) +
                                                int(np.prod(shapes[nd["y"]])))
        per_node.append((nd["y"], op, mac, nbytes))
    return dict(params=params, macs=macs, per_node=per_node, shapes=shapes)
