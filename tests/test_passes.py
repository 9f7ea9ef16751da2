"""Graph-level passes (Section 3.4 of the paper): structure of the rewritten graphs, and
equivalence of the rewritten graph with the graph it came from, both evaluated by the CPU oracle
(the operator-by-operator graph by the operators' definitions)."""
import collections

import numpy as np
import pytest

import oracle
import oracle.chain
import workloads
from util import REL_TOL, rel_err

passes = pytest.importorskip("paper_2008_08272_amd.passes")


def ops(model):
    return collections.Counter(nd["op"] for nd in model["graph"])


def test_oracle_batchnorm_matches_torch_float64():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(5)
    x = rng.standard_normal((3, 7, 5, 4)).astype(np.float32)
    g, b, m = (rng.standard_normal(7).astype(np.float32) for _ in range(3))
    v = rng.uniform(0.5, 2.0, 7).astype(np.float32)
    ref = torch.nn.functional.batch_norm(torch.from_numpy(x).double(), torch.from_numpy(m).double(),
                                         torch.from_numpy(v).double(), torch.from_numpy(g).double(),
                                         torch.from_numpy(b).double(), training=False, eps=1e-5).numpy()
    got = oracle.chain.batchnorm(x, g, b, m, v, 1e-5)
    assert np.abs(got - ref).max() <= 1e-12 * np.abs(ref).max()
    # worked value: x = 3, mean 1, var 4 - eps, scale 2, bias -1  ->  (3 - 1) / 2 * 2 - 1 = 1
    one = oracle.chain.batchnorm(np.full((1, 1, 1, 1), 3, np.float32), [2.0], [-1.0], [1.0], [4.0 - 1e-5], 1e-5)
    assert abs(one.item() - 1.0) < 1e-12


def test_small_cnn_rewrites_to_the_fused_chain():
    raw = workloads.small_cnn_unfused()
    opt = passes.optimize(raw)
    fused = workloads.small_cnn()
    assert [nd["op"] for nd in opt["graph"]] == [nd["op"] for nd in fused["graph"]]
    assert ops(opt) == collections.Counter(conv=2, maxpool=2, reshape=1, gemm=1)
    g = opt["graph"][-1]
    assert (g["a"], g["b"], g["c"], g["alpha"], g["beta"], g["transA"], g["transB"]) == ("flat", "wg", "bg", 1.0, 1.0, 0, 0)
    assert all(nd["relu"] for nd in opt["graph"] if nd["op"] == "conv")
    assert opt["graph"][0]["x"] == "x"                       # the Identity is gone
    assert set(opt["weights"]) == set(fused["weights"])
    _, e_raw = oracle.chain.run(raw)
    _, e_opt = oracle.chain.run(opt)
    assert rel_err(e_opt["logits"], e_raw["logits"]) <= 1e-6
    # the input graph is left untouched
    assert ops(raw)["relu"] == 2 and ops(raw)["identity"] == 1


def test_resnet50_rewrites_to_one_call_per_convolution():
    raw = workloads.resnet50_unfused(1, image=32)
    assert ops(raw) == collections.Counter(conv=53, batchnorm=53, relu=49, add=16, maxpool=1, avgpool=1,
                                           reshape=1, gemm=1)
    opt = passes.optimize(raw)
    assert ops(opt) == collections.Counter(conv=53, maxpool=1, avgpool=1, reshape=1, gemm=1)
    convs = [nd for nd in opt["graph"] if nd["op"] == "conv"]
    assert sum(1 for nd in convs if nd["residual"]) == 16
    assert sum(1 for nd in convs if nd["relu"]) == 49
    assert all(nd["b"] for nd in convs)
    # no BatchNorm parameter survives, every tensor a node names exists when the node runs
    assert not [k for k in opt["weights"] if k.endswith(("_gamma", "_beta", "_mean", "_var"))]
    known = set(opt["inputs"]) | set(opt["weights"])
    for nd in opt["graph"]:
        for f in ("x", "w", "b", "residual", "a", "c"):
            if nd.get(f):
                assert nd[f] in known, (nd["y"], f, nd[f])
        known.add(nd["y"])
    _, e_raw = oracle.chain.run(raw)
    _, e_opt = oracle.chain.run(opt)
    assert rel_err(e_opt["logits"], e_raw["logits"]) <= 1e-5
    # the folded filters equal the ones the workload generator folds from its double-precision
    # draws up to the fp32 rounding of the BatchNorm parameters
    pre = workloads.resnet50(1, image=32)
    w_opt = opt["weights"][convs[0]["w"]]
    assert rel_err(w_opt, pre["weights"]["stem_w"]) <= 1e-6


def test_fold_batchnorm_formula_with_a_conv_bias():
    rng = np.random.default_rng(9)
    W = rng.standard_normal((4, 3, 3, 3)).astype(np.float32)
    b = rng.standard_normal(4).astype(np.float32)
    g, beta, mean = (rng.standard_normal(4).astype(np.float32) for _ in range(3))
    var = rng.uniform(0.5, 2.0, 4).astype(np.float32)
    X = rng.standard_normal((2, 3, 6, 5)).astype(np.float32)
    m = dict(name="t", inputs={"x": X}, output="y",
             weights=dict(W=W, b=b, g=g, beta=beta, mean=mean, var=var),
             graph=[workloads.conv_node("x", "W", "b", "c", pads=(1, 1, 1, 1)),
                    workloads.batchnorm_node("c", "g", "beta", "mean", "var", "y", 1e-3)])
    f = passes.fold_batchnorm(m)
    assert [nd["op"] for nd in f["graph"]] == ["conv"]
    s = g.astype(np.float64) / np.sqrt(var.astype(np.float64) + 1e-3)
    assert np.array_equal(f["weights"][f["graph"][0]["w"]], (W.astype(np.float64) * s[:, None, None, None]).astype(np.float32))
    assert np.array_equal(f["weights"][f["graph"][0]["b"]], ((b.astype(np.float64) - mean) * s + beta).astype(np.float32))
    _, e0 = oracle.chain.run(m)
    _, e1 = oracle.chain.run(f)
    assert rel_err(e1["y"], e0["y"]) <= 1e-6


def test_patterns_that_must_not_fire():
    rng = np.random.default_rng(10)
    X = rng.standard_normal((1, 2, 4, 4)).astype(np.float32)
    W = rng.standard_normal((2, 2, 1, 1)).astype(np.float32)
    # the convolution's result has a second consumer: neither the Relu nor the Add may be folded into it
    m = dict(name="t", inputs={"x": X}, weights={"W": W}, output="out",
             graph=[workloads.conv_node("x", "W", None, "c"),
                    workloads.relu_node("c", "r"),
                    workloads.add_node("c", "r", "out")])
    o = passes.optimize(m)
    assert [nd["op"] for nd in o["graph"]] == ["conv", "relu", "add"]
    # MatMul whose product is used twice stays a MatMul; batched MatMul is never a Gemm
    A = rng.standard_normal((3, 4)).astype(np.float32)
    Bm = rng.standard_normal((4, 5)).astype(np.float32)
    C = rng.standard_normal((1, 5)).astype(np.float32)
    m = dict(name="t", inputs={"a": A}, weights={"B": Bm, "C": C}, output="z",
             graph=[workloads.matmul_node("a", "B", "p"), workloads.add_node("p", "C", "q"),
                    workloads.add_node("p", "q", "z")])
    assert [nd["op"] for nd in passes.matmul_add_to_gemm(m)["graph"]] == ["matmul", "add", "add"]
    A3 = rng.standard_normal((2, 3, 4)).astype(np.float32)
    m = dict(name="t", inputs={"a": A3}, weights={"B": Bm, "C": C}, output="q",
             graph=[workloads.matmul_node("a", "B", "p"), workloads.add_node("p", "C", "q")])
    assert [nd["op"] for nd in passes.matmul_add_to_gemm(m)["graph"]] == ["matmul", "add"]
    # C on the left of the Add works too, and (M,1) column bias is accepted
    Cc = rng.standard_normal((3, 1)).astype(np.float32)
    m = dict(name="t", inputs={"a": A}, weights={"B": Bm, "C": Cc}, output="q",
             graph=[workloads.matmul_node("a", "B", "p"), workloads.add_node("C", "p", "q")])
    g = passes.matmul_add_to_gemm(m)
    assert [nd["op"] for nd in g["graph"]] == ["gemm"]
    _, e0 = oracle.chain.run(m)
    _, e1 = oracle.chain.run(g)
    assert rel_err(e1["q"], e0["q"]) <= 1e-6


def test_infer_shapes_matches_the_oracle_chain():
    for m in (workloads.small_cnn_unfused(), workloads.resnet50_unfused(2, image=64)):
        sh = passes.infer_shapes(m)
        env, _ = oracle.chain.run(m)
        for nd in m["graph"]:
            assert sh[nd["y"]] == tuple(env[nd["y"]].shape), nd["y"]
    bad = workloads.small_cnn_unfused()
    bad["graph"][7] = workloads.reshape_node("p2", "flat", (1, 255))
    with pytest.raises(ValueError):
        passes.infer_shapes(bad)


def test_constant_propagation_normalises_adds_and_folds_constants():
    """Section 3.4's Add normalisation rules: after the pass every constant of the chain has met
    in one constant, operators on constants only are gone, and the graph computes the same
    function (up to the rounding of the reassociated fp32 sums)."""
    raw = workloads.constant_adds()
    assert ops(raw) == collections.Counter(add=9, relu=2)
    opt = passes.propagate_constants(raw)
    assert ops(opt) == collections.Counter(add=4, relu=1)
    consts = [nd for nd in opt["graph"] if nd["op"] == "add" and nd["b"] in opt["weights"]]
    assert len(consts) == 1 and consts[0]["y"] == "out" and len(opt["weights"]) == 1
    assert not any(nd["op"] == "add" and nd["a"] in opt["weights"] for nd in opt["graph"])
    # the merged constant is the sum of all constants of the original chain, broadcast
    w = raw["weights"]
    k2 = np.maximum(w["c5"].astype(np.float64) + w["c6"], 0)
    want = w["c1"].astype(np.float64) + w["c2"] + k2 + w["c3"] + w["c4"]
    got = opt["weights"][consts[0]["b"]]
    assert got.dtype == np.float32 and got.shape == want.shape
    assert np.abs(got - want).max() <= 8 * 2.0 ** -24 * np.abs(want).max()
    _, e_raw = oracle.chain.run(raw)
    _, e_opt = oracle.chain.run(opt)
    assert rel_err(e_opt["out"], e_raw["out"]) <= 1e-6
    assert ops(raw) == collections.Counter(add=9, relu=2)          # the input graph is left untouched


@pytest.mark.parametrize("rule", ["c+x", "(x+c1)+c2", "(x+c)+y", "x+(y+c)", "(x+c1)+(y+c2)", "shared inner"])
def test_each_add_normalisation_rule(rule):
    rng = np.random.default_rng(11)
    x, y = rng.standard_normal((2, 3, 4)).astype(np.float32), rng.standard_normal((2, 3, 4)).astype(np.float32)
    c1, c2 = rng.standard_normal((3, 1)).astype(np.float32), rng.standard_normal((4,)).astype(np.float32)
    A = workloads.add_node
    graphs = {
        "c+x": [A("c1", "x", "out")],
        "(x+c1)+c2": [A("x", "c1", "t"), A("t", "c2", "out")],
        "(x+c)+y": [A("x", "c1", "t"), A("t", "y", "out")],
        "x+(y+c)": [A("y", "c1", "t"), A("x", "t", "out")],
        "(x+c1)+(y+c2)": [A("x", "c1", "t"), A("y", "c2", "u"), A("t", "u", "out")],
        "shared inner": [A("x", "c1", "t"), A("t", "c2", "u"), A("t", "u", "out")],     # t has two readers: it stays
    }
    raw = dict(name=rule, inputs={"x": x, "y": y}, weights={"c1": c1, "c2": c2}, graph=graphs[rule], output="out")
    opt = passes.propagate_constants(raw)
    g = opt["graph"]
    if rule == "c+x":
        assert [(n["a"], n["b"]) for n in g] == [("x", "c1")]
    elif rule == "(x+c1)+c2":
        assert len(g) == 1 and g[0]["a"] == "x" and np.array_equal(opt["weights"][g[0]["b"]], c1 + c2)
    elif rule in ("(x+c)+y", "x+(y+c)"):
        assert len(g) == 2 and {g[0]["a"], g[0]["b"]} == {"x", "y"} and (g[1]["a"], g[1]["b"]) == (g[0]["y"], "c1")
    elif rule == "(x+c1)+(y+c2)":
        assert len(g) == 2 and (g[0]["a"], g[0]["b"]) == ("x", "y") and np.array_equal(opt["weights"][g[1]["b"]], c1 + c2)
    else:
        # t = x + c1 is read twice and is left alone; u = t + c2 is read once: t + (t + c2) -> (t + t) + c2
        assert len(g) == 3 and (g[0]["a"], g[0]["b"], g[0]["y"]) == ("x", "c1", "t")
        assert (g[1]["a"], g[1]["b"]) == ("t", "t") and (g[2]["a"], g[2]["b"], g[2]["y"]) == (g[1]["y"], "c2", "out")
    _, e_raw = oracle.chain.run(raw)
    _, e_opt = oracle.chain.run(opt)
    assert rel_err(e_opt["out"], e_raw["out"]) <= 1e-6
    assert passes.infer_shapes(opt)["out"] == passes.infer_shapes(raw)["out"]
