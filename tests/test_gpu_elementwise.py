"""GPU parity of the element-wise, reduction and softmax entry points against the CPU oracle
(numpy, double).  Add / Relu / LeakyRelu / Abs round once from an exact or correctly rounded
result, so they are compared bit for bit on data where double rounding cannot occur; sums and
softmax within the fp32 tolerance."""
import numpy as np
import pytest

import workloads
from oracle import elementwise as ew
from util import REL_TOL, rel_err

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lib():
    import paper_2008_08272_amd as p
    assert torch.cuda.is_available(), "these tests need the GPU"
    return p


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def announce(*what):
    print("CASE", *what, flush=True)


ADD_SHAPES = [
    ((3, 4, 5), (3, 4, 5)),                   # the paper's running example
    ((2, 64, 9, 7), (2, 64, 9, 7)),           # odd element count: scalar tail
    ((2, 64, 12, 12), (64, 1, 1)),            # per-channel bias
    ((2, 64, 12, 12), (1, 64, 1, 1)),
    ((37, 1000), (1000,)),                    # row vector
    ((37, 1000), (37, 1)),                    # column vector
    ((5, 1, 7), (1, 6, 1)),                   # both operands broadcast
    ((4,), (3, 2, 4)),
    ((2, 3), ()),                             # scalar
    ((1,), (1,)),
    ((8, 3, 1, 16, 1, 4), (1, 3, 5, 1, 2, 4)),
    ((1 << 20,), (1 << 20,)),                 # several grid-stride rounds
    ((1031, 517), (1031, 517)),
]


@pytest.mark.parametrize("sa,sb", ADD_SHAPES)
def test_add_bit_exact_on_small_integers_and_within_tolerance(lib, sa, sb):
    announce("add", sa, sb)
    rng = np.random.default_rng(11)
    a = rng.integers(-1000, 1000, sa).astype(np.float32)
    b = rng.integers(-1000, 1000, sb).astype(np.float32)
    ref = ew.add(a, b)
    got = host(lib.onnx_add(dev(a), dev(b)))
    assert got.shape == ref.shape
    assert np.array_equal(got, ref.astype(np.float32))
    a = rng.uniform(-1, 1, sa).astype(np.float32)
    b = rng.uniform(-1, 1, sb).astype(np.float32)
    ref = ew.add(a, b)
    got = host(lib.onnx_add(dev(a), dev(b)))
    assert np.array_equal(got, ref.astype(np.float32))       # |a|,|b| < 1 with 24-bit mantissas: the double sum is exact
    assert rel_err(got, ref) <= REL_TOL


@pytest.mark.parametrize("n", [1, 3, 4, 255, 1024, 100003, (1 << 22) + 5])
def test_unary_bit_exact(lib, n):
    announce("unary", n)
    rng = np.random.default_rng(12)
    x = rng.standard_normal(n).astype(np.float32)
    x[::7] = 0.0
    xd = dev(x)
    assert np.array_equal(host(lib.onnx_relu(xd)), ew.relu(x).astype(np.float32))
    assert np.array_equal(host(lib.onnx_abs(xd)), ew.absolute(x).astype(np.float32))
    for alpha in (0.01, 0.1, 0.3):
        assert np.array_equal(host(lib.onnx_leakyrelu(xd, alpha)), ew.leakyrelu(x, alpha).astype(np.float32))
    # a view that is not 16-byte aligned takes the scalar path
    if n > 8:
        sub = xd[1:]
        assert sub.is_contiguous() and sub.data_ptr() % 16 == 4
        assert np.array_equal(host(lib.onnx_relu(sub)), ew.relu(x[1:]).astype(np.float32))
        assert np.array_equal(host(lib.onnx_abs(sub)), ew.absolute(x[1:]).astype(np.float32))
        assert np.array_equal(host(lib.onnx_leakyrelu(sub, 0.2)), ew.leakyrelu(x[1:], 0.2).astype(np.float32))


REDUCE_CASES = [
    # shape, axes, keepdims
    ((7,), None, 1), ((1000,), [0], 0), ((33, 65), [1], 0), ((33, 65), [0], 1), ((33, 65), None, 0),
    ((4, 5, 6, 7), [1, 3], 1), ((4, 5, 6, 7), [0, 2], 0), ((4, 5, 6, 7), [-1], 1), ((4, 5, 6, 7), [1, 2], 0),
    ((2, 3, 4, 5, 6), [0, 2, 4], 0), ((2, 3, 4, 5, 6), [1, 3], 1),
    ((32, 2048, 7, 7), [2, 3], 1),            # global sum pooling
    ((32, 1000), [1], 0), ((32, 1000), [0], 1),
    ((1 << 21,), None, 0),                    # one output, long sum (two stages when a workspace is set)
    ((3, 1 << 18), [1], 0),
    ((1 << 16, 5), [0], 0),                   # few outputs, innermost extent kept
    ((6, 1, 9), [1], 0), ((6, 1, 9), [1], 1), # reducing a unit extent
]


@pytest.mark.parametrize("use_ws", [False, True])
@pytest.mark.parametrize("shape,axes,keep", REDUCE_CASES)
def test_reducesum_matches_oracle(lib, shape, axes, keep, use_ws):
    announce("reducesum", shape, axes, keep, use_ws)
    ws = torch.empty(8 << 20, dtype=torch.uint8, device="cuda") if use_ws else None
    lib.onnx_set_workspace(ws)
    try:
        rng = np.random.default_rng(13)
        x = rng.integers(-8, 9, shape).astype(np.float32)       # every partial sum is an exact integer
        got = host(lib.onnx_reducesum(dev(x), axes, keep))
        ref = ew.reducesum(x, axes, keep)
        assert got.shape == ref.shape
        assert np.array_equal(got, ref.astype(np.float32))
        x = rng.standard_normal(shape).astype(np.float32)
        got = host(lib.onnx_reducesum(dev(x), axes, keep))
        ref = ew.reducesum(x, axes, keep)
        scale = ew.reducel1(x, axes, keep)                      # sum of |x|: the scale of the rounding bound
        count = x.size // max(ref.size, 1)
        assert (np.abs(got - ref) <= (count + 2) * 2.0 ** -24 * scale + 1e-30).all()
        assert rel_err(got, ref) <= REL_TOL
    finally:
        torch.cuda.synchronize()
        lib.onnx_set_workspace(None)


@pytest.mark.parametrize("shape,axis", [((1, 5), 1), ((32, 1000), 1), ((32, 1000), -1), ((32, 1000), 0), ((7, 1025), 1),
                                        ((3, 5000), 1), ((4, 9, 6), 1), ((4, 9, 6), 0), ((2, 3, 4, 5), 2), ((513,), 0),
                                        ((6, 1), 1), ((300, 3, 257), 1)])
def test_softmax_matches_oracle(lib, shape, axis):
    announce("softmax", shape, axis)
    rng = np.random.default_rng(14)
    for scale in (1.0, 30.0):
        x = (rng.standard_normal(shape) * scale).astype(np.float32)
        got = host(lib.onnx_softmax(dev(x), axis))
        ref = ew.softmax(x, axis)
        assert got.shape == ref.shape
        assert rel_err(got, ref) <= REL_TOL
        assert np.abs(got.astype(np.float64).sum(axis=axis) - 1.0).max() <= 1e-5
        # element-wise: the fp32 subtraction x - max rounds by up to 2^-24 |x - max|, which exp turns
        # into that relative error; plus a few roundings of exp, the sum and the division
        depth = np.abs(x.astype(np.float64) - x.astype(np.float64).max(axis=axis, keepdims=True))
        assert (np.abs(got - ref) <= (depth * 2.0 ** -23 + 4e-6) * ref + 1e-37).all()
    big = np.array([[1000.0, 1000.0, -1000.0]], np.float32)
    assert host(lib.onnx_softmax(dev(big), 1)).tolist() == [[0.5, 0.5, 0.0]]


def test_zero_sized_and_errors(lib):
    announce("elementwise degenerate")
    e = torch.empty((0, 4), dtype=torch.float32, device="cuda")
    assert lib.onnx_add(e, torch.ones(4, device="cuda")).shape == (0, 4)
    assert lib.onnx_relu(e).shape == (0, 4)
    assert lib.onnx_softmax(e, 1).shape == (0, 4)
    z = host(lib.onnx_reducesum(e, [0], 0))                  # empty sum
    assert z.tolist() == [0.0, 0.0, 0.0, 0.0]
    y = torch.full((4,), 7.0, device="cuda")
    with pytest.raises(lib.OnnxHipError):
        lib.onnx_add(torch.ones((2, 3), device="cuda"), torch.ones((4,), device="cuda"), out=y)
    with pytest.raises(lib.OnnxHipError):
        lib.onnx_reducesum(torch.ones((2, 3), device="cuda"), [2], 1)
    assert host(y).tolist() == [7.0] * 4


def test_classifier_head_graph(lib):
    """LeakyRelu -> MatMul + Add -> Softmax, ReduceL1 (decomposed into Abs + ReduceSum) and a
    column ReduceSum through passes + runner, against the oracle on the original graph."""
    announce("classifier head")
    from oracle import chain
    from paper_2008_08272_amd import passes
    from paper_2008_08272_amd.runner import GraphRunner
    raw = workloads.classifier_head(32)
    with pytest.raises(NotImplementedError):
        GraphRunner(raw)                                     # ReduceL1 has no kernel before the decomposition
    opt = passes.optimize(raw)
    assert [nd["op"] for nd in opt["graph"]] == ["leakyrelu", "gemm", "softmax", "abs", "reducesum", "reducesum"]
    _, exact = chain.run(raw)
    r = GraphRunner(opt)
    r.run()
    torch.cuda.synchronize()
    for name in ("act", "logits", "prob", "l1", "colsum"):
        got = r.t[name].cpu().numpy()
        assert got.shape == exact[name].shape, name
        assert rel_err(got, exact[name]) <= REL_TOL, name
