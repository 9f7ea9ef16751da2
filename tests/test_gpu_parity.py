"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, same seeded inputs.

Floating outputs: max_i |g_i - r_i| / max(|r_i|, rms(r)) <= 1e-4 against the fp64 oracle, and
the a-priori component-wise fp32 rounding bound where the oracle supplies the scale.
MaxPool values and indices, delta-kernel convolutions and small-integer data: bit-exact.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads
from util import REL_TOL, rel_err, within_rounding_bound

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lib():
    import paper_2008_08272_amd as p
    assert torch.cuda.is_available(), "these tests need the GPU"
    return p


@pytest.fixture(scope="module", params=["no_workspace", "workspace"], autouse=True)
def workspace(request, lib):
    """Every parity case runs twice: without scratch memory (no split-K) and with a 64 MiB
    workspace (products with few output tiles then split their K range)."""
    if request.param == "workspace":
        ws = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
        lib.onnx_set_workspace(ws)
    else:
        lib.onnx_set_workspace(None)
    yield request.param
    torch.cuda.synchronize()
    lib.onnx_set_workspace(None)


def dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def announce(*what):
    print("CASE", *what, flush=True)


_ORACLE_CACHE = {}


def cached(key, fn):
    """Every case runs with and without a workspace; the oracle's result for a large case is
    computed once and kept for the second pass."""
    if key not in _ORACLE_CACHE:
        _ORACLE_CACHE[key] = fn()
    return _ORACLE_CACHE[key]


# ------------------------------------------------------------------------------ Gemm

GEMM_SHAPES = [
    # M, N, K : several tiles plus ragged tails in every dimension, both tile shapes, vec4 and scalar
    (1, 1, 1), (3, 5, 7), (64, 64, 16), (65, 63, 17), (200, 150, 70), (130, 257, 129),
    (256, 384, 64), (300, 520, 36), (1, 1000, 2048), (32, 1000, 2048), (513, 1025, 40),
    (2048, 1536, 20),
]


@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
@pytest.mark.parametrize("transA,transB", [(0, 0), (0, 1), (1, 0), (1, 1)])
def test_gemm_matches_oracle(lib, M, N, K, transA, transB):
    announce("gemm", M, N, K, transA, transB)
    rng = np.random.default_rng([M, N, K, transA, transB])
    A = rng.uniform(-1, 1, (K, M) if transA else (M, K)).astype(np.float32)
    B = rng.uniform(-1, 1, (N, K) if transB else (K, N)).astype(np.float32)
    cshape = [(1, N), (M, 1), (M, N), (N,), (), (1, 1)][(M + N + K + transA) % 6]
    C = rng.uniform(-1, 1, cshape).astype(np.float32)
    alpha, beta = 0.75, -1.25
    relu = bool((M + K) % 2)
    ref, S = oracle.gemm(A, B, C, alpha, beta, transA, transB, relu=relu, want_scale=True)
    got = host(lib.onnx_gemm(dev(A), dev(B), dev(C), alpha, beta, transA, transB, act=int(relu)))
    assert got.shape == ref.shape
    assert rel_err(got, ref) <= REL_TOL
    if not relu:
        assert within_rounding_bound(got, ref, S, K + 2)


def test_gemm_no_bias_and_defaults(lib):
    announce("gemm no bias")
    rng = np.random.default_rng(3)
    A = rng.uniform(-1, 1, (70, 90)).astype(np.float32)
    B = rng.uniform(-1, 1, (90, 50)).astype(np.float32)
    got = host(lib.onnx_gemm(dev(A), dev(B)))
    assert rel_err(got, oracle.gemm(A, B)) <= REL_TOL


@pytest.mark.parametrize("M,N,K", [(257, 383, 96), (128, 128, 512), (1000, 70, 33)])
def test_gemm_small_integers_bit_exact(lib, M, N, K):
    """With inputs in {-4..4} every partial sum is an exactly representable integer, so any
    summation order gives the same bits: a dropped, duplicated or misplaced k shows up."""
    announce("gemm integer", M, N, K)
    rng = np.random.default_rng([M, N, K])
    A = rng.integers(-4, 5, (M, K)).astype(np.float32)
    B = rng.integers(-4, 5, (N, K)).astype(np.float32)
    C = rng.integers(-4, 5, (1, N)).astype(np.float32)
    ref = oracle.gemm(A, B, C, 1.0, 1.0, 0, 1)
    got = host(lib.onnx_gemm(dev(A), dev(B), dev(C), 1.0, 1.0, 0, 1))
    assert np.array_equal(got.astype(np.float64), ref)
    Bt = np.ascontiguousarray(B.T)
    got2 = host(lib.onnx_gemm(dev(np.ascontiguousarray(A.T)), dev(Bt), dev(C), 1.0, 1.0, 1, 0))
    assert np.array_equal(got2.astype(np.float64), ref)


def test_gemm_sweep_1024_full(lib):
    announce("gemm sweep 1024")
    c = workloads.gemm_case(1024)
    ref, S = oracle.gemm(c["A"], c["B"], c["C"], 1.0, 1.0, 0, 1, want_scale=True)
    got = host(lib.onnx_gemm(dev(c["A"]), dev(c["B"]), dev(c["C"]), 1.0, 1.0, 0, 1))
    assert rel_err(got, ref) <= REL_TOL
    assert within_rounding_bound(got, ref, S, 1024 + 2)


@pytest.mark.parametrize("n", [2048, 4096])
def test_gemm_sweep_full_size_whole_output(lib, n):
    """The launches the benchmark times (4096: the 256 x 256 tile, one workgroup per CU), every
    output element compared with the oracle, without and with the fused Relu."""
    announce("gemm sweep full", n)
    c = workloads.gemm_case(n)
    ref, S = cached(("gemm_sweep", n), lambda: oracle.gemm(c["A"], c["B"], c["C"], 1.0, 1.0, 0, 1, want_scale=True))
    a, b, cc = dev(c["A"]), dev(c["B"]), dev(c["C"])
    got = host(lib.onnx_gemm(a, b, cc, 1.0, 1.0, 0, 1))
    if n == 4096:
        assert lib.onnx_last_launch().startswith("contraction 256x256x16 waves 4x4x1 A=KC/4 B=KC/4"), lib.onnx_last_launch()
    assert rel_err(got, ref) <= REL_TOL
    assert within_rounding_bound(got, ref, S, n + 2)
    got_r = host(lib.onnx_gemm(a, b, cc, 1.0, 1.0, 0, 1, act=1))
    assert rel_err(got_r, np.maximum(ref, 0)) <= REL_TOL


# ------------------------------------------------------------------------------ MatMul

@pytest.mark.parametrize("sa,sb", [
    ((5, 4), (4, 6)), ((3, 2, 50, 40), (2, 40, 60)), ((2, 70, 33), (3, 1, 33, 65)), ((40,), (40, 6)),
    ((50, 40), (40,)), ((40,), (40,)), ((3, 1, 5, 4), (1, 2, 4, 6)), ((2, 3, 130, 36), (36, 200)),
    ((4,), (2, 3, 4, 6)), ((2, 3, 5, 4), (4,)), ((2, 2, 2, 2, 2, 9, 8), (2, 1, 2, 8, 7)),
])
def test_matmul_matches_oracle(lib, sa, sb):
    announce("matmul", sa, sb)
    rng = np.random.default_rng(len(sa) * 100 + len(sb))
    A = rng.uniform(-1, 1, sa).astype(np.float32)
    B = rng.uniform(-1, 1, sb).astype(np.float32)
    ref = oracle.matmul(A, B)
    got = host(lib.onnx_matmul(dev(A), dev(B)))
    assert got.shape == ref.shape
    assert rel_err(got, ref) <= REL_TOL


def test_matmul_attribute_sweep_heads(lib):
    """[8,12,512,64] x [8,12,64,512]: all 96 products compared."""
    announce("matmul heads full")
    c = workloads.attr_sweep_case("matmul_heads")
    ref, S = cached("matmul_heads", lambda: oracle.matmul(c["A"], c["B"], want_scale=True))
    got = host(lib.onnx_matmul(dev(c["A"]), dev(c["B"])))
    assert got.shape == (8, 12, 512, 512)
    assert rel_err(got, ref) <= REL_TOL
    assert within_rounding_bound(got, ref, S, 64)


def test_matmul_attribute_sweep_projection(lib):
    """[8,512,768] x [768,3072]: the whole [8,512,3072] result compared."""
    announce("matmul proj full")
    c = workloads.attr_sweep_case("matmul_proj")
    ref, S = cached("matmul_proj", lambda: oracle.matmul(c["A"], c["B"], want_scale=True))
    got = host(lib.onnx_matmul(dev(c["A"]), dev(c["B"])))
    assert got.shape == (8, 512, 3072)
    assert rel_err(got, ref) <= REL_TOL
    assert within_rounding_bound(got, ref, S, 768)


# ------------------------------------------------------------------------------ Conv

CONV_CASES = [
    # N, C, H, W, M, kH, kW, pads, strides, dilations, group      (path the selector takes)
    (2, 4, 7, 6, 6, 3, 2, (1, 0, 2, 1), (2, 1), (1, 2), 2),          # direct (tiny groups)
    (1, 1, 28, 28, 8, 5, 5, (2, 2, 2, 2), (1, 1), (1, 1), 1),        # direct (M = 8)
    (1, 8, 14, 14, 16, 5, 5, (2, 2, 2, 2), (1, 1), (1, 1), 1),       # matrix cores, K = 200
    (3, 16, 19, 23, 40, 3, 3, (1, 1, 1, 1), (1, 1), (1, 1), 1),      # ragged tiles, several images per tile
    (2, 3, 37, 41, 64, 7, 7, (3, 3, 3, 3), (2, 2), (1, 1), 1),       # K = 147 (scalar filter loads)
    (2, 32, 20, 20, 48, 3, 3, (2, 0, 1, 3), (2, 3), (2, 1), 2),      # asymmetric pads, stride, dilation, 2 groups
    (2, 64, 12, 12, 96, 1, 1, (0, 0, 0, 0), (1, 1), (1, 1), 1),      # pointwise fast path (16-byte loads)
    (2, 64, 9, 7, 96, 1, 1, (0, 0, 0, 0), (1, 1), (1, 1), 1),        # pointwise, P = 63 (scalar loads)
    (2, 64, 12, 12, 96, 1, 1, (0, 0, 0, 0), (2, 2), (1, 1), 1),      # strided 1x1 (projection shortcut)
    (3, 20, 13, 11, 40, 1, 1, (0, 0, 0, 0), (3, 2), (1, 1), 1),      # strided 1x1, unequal strides, odd extents
    (2, 64, 14, 14, 128, 1, 1, (0, 0, 0, 0), (2, 2), (1, 1), 2),     # strided 1x1 with 2 groups
    (2, 64, 12, 12, 64, 1, 1, (1, 1, 1, 1), (1, 1), (1, 1), 4),      # padded 1x1 with 4 groups
    (1, 24, 30, 30, 160, 3, 3, (2, 2, 2, 2), (1, 1), (2, 2), 1),     # dilated, > 128 rows
    (5, 40, 15, 15, 200, 3, 3, (1, 1, 1, 1), (1, 1), (1, 1), 1),     # 128x128 tiles with tails
    (4, 6, 10, 10, 6, 3, 3, (1, 1, 1, 1), (1, 1), (1, 1), 6),        # depthwise
    (1, 16, 5, 5, 32, 5, 5, (0, 0, 0, 0), (1, 1), (1, 1), 1),        # output 1x1
    # 3x3 with few channels per group (row-strip kernel: one wavefront per 8 rows x 64 columns)
    (2, 5, 21, 150, 5, 3, 3, (1, 1, 1, 1), (1, 1), (1, 1), 5),       # depthwise, 3 column chunks, ragged last strip
    (2, 6, 21, 40, 6, 3, 3, (1, 1, 1, 1), (2, 1), (1, 1), 6),        # depthwise, vertical stride 2, a row per wavefront: one load per row
    (2, 6, 23, 70, 12, 3, 3, (0, 2, 1, 0), (2, 2), (1, 1), 3),       # vertical stride 2, 2 channels per group, asymmetric pads
    (1, 4, 19, 66, 4, 3, 3, (2, 2, 2, 2), (1, 3), (2, 2), 4),        # vertical dilation 2, horizontal stride 3
    (3, 8, 9, 9, 8, 3, 3, (1, 1, 1, 1), (3, 1), (1, 1), 8),          # vertical stride 3: falls back to the plane kernel
    (2, 4, 2, 2, 4, 3, 3, (1, 1, 1, 1), (1, 1), (1, 1), 4),          # plane smaller than the filter
    (2, 6, 17, 64, 6, 3, 3, (1, 1, 1, 1), (1, 1), (1, 1), 6),        # full-width rows: neighbour lanes supply the side taps
    (2, 4, 9, 64, 4, 3, 3, (0, 1, 2, 2), (2, 1), (1, 1), 4),         # 65 output columns: two chunks, plain loads
    (1, 8, 20, 33, 16, 3, 3, (2, 1, 0, 0), (1, 1), (2, 1), 4),       # right pad 0, vertical dilation 2, 2 channels per group
]


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_matches_oracle(lib, case):
    announce("conv", case)
    N, C, H, W, M, kH, kW, pads, st, dl, g = case
    rng = np.random.default_rng(list(case[:7]) + [g])
    X = rng.uniform(-1, 1, (N, C, H, W)).astype(np.float32)
    Wt = rng.uniform(-1, 1, (M, C // g, kH, kW)).astype(np.float32)
    Bv = rng.uniform(-1, 1, (M,)).astype(np.float32)
    K = (C // g) * kH * kW
    ref, S = oracle.conv(X, Wt, Bv, pads, st, dl, g, want_scale=True)
    got = host(lib.onnx_conv(dev(X), dev(Wt), dev(Bv), pads, st, dl, g))
    assert got.shape == ref.shape
    assert rel_err(got, ref) <= REL_TOL
    assert within_rounding_bound(got, ref, S, K + 1)
    # fused residual + Relu, and no bias
    R = rng.uniform(-1, 1, ref.shape).astype(np.float32)
    ref2 = oracle.conv(X, Wt, None, pads, st, dl, g, residual=R, relu=True)
    got2 = host(lib.onnx_conv(dev(X), dev(Wt), None, pads, st, dl, g, residual=dev(R), act=1))
    assert rel_err(got2, ref2) <= REL_TOL
    assert (got2 >= 0).all()


RESIDENT_CASES = [
    # N, H, W, M, pads, resident: 7x7 stride-2 convolutions of 3-channel images.  With two or more 8x16 output tiles
    # per CU and filter block the filters stay in registers; below that the gathering contraction kernel runs.
    (90, 37, 41, 64, (3, 3, 3, 3), True),         # ragged tiles in both directions
    (6, 224, 224, 64, (3, 3, 3, 3), True),        # ResNet-50's stem: 14 x 7 whole tiles per image
    (32, 64, 50, 96, (0, 2, 5, 1), True),         # asymmetric pads, 96 filters: the second filter block is half empty
    (18, 23, 130, 130, (6, 6, 6, 6), True),       # pads as large as they may be, three filter blocks, two rows of tiles
    (512, 7, 7, 32, (0, 0, 0, 0), True),          # a single output position per image
    (1, 224, 224, 64, (3, 3, 3, 3), False),       # the stem at batch 1: 98 tiles
    (5, 224, 224, 64, (3, 3, 3, 3), False),       # 490 tiles: the last batch below the switch
    (2, 37, 41, 64, (3, 3, 3, 3), False),
]


@pytest.mark.parametrize("case", RESIDENT_CASES)
def test_conv_resident_filters_matches_oracle(lib, case):
    N, H, W, M, pads, resident = case
    announce("conv resident", case)
    rng = np.random.default_rng([N, H, W, M])
    X = rng.uniform(-1, 1, (N, 3, H, W)).astype(np.float32)
    Wt = rng.uniform(-1, 1, (M, 3, 7, 7)).astype(np.float32)
    Bv = rng.uniform(-1, 1, (M,)).astype(np.float32)
    ref, S = oracle.conv(X, Wt, Bv, pads, (2, 2), (1, 1), 1, want_scale=True)
    got = host(lib.onnx_conv(dev(X), dev(Wt), dev(Bv), pads, (2, 2), (1, 1), 1))
    assert lib.onnx_last_launch().startswith("conv_resident 64x128x147" if resident else "contraction "), lib.onnx_last_launch()
    assert got.shape == ref.shape
    assert rel_err(got, ref) <= REL_TOL
    assert within_rounding_bound(got, ref, S, 147 + 1)
    R = rng.uniform(-1, 1, ref.shape).astype(np.float32)
    ref2 = oracle.conv(X, Wt, None, pads, (2, 2), (1, 1), 1, residual=R, relu=True)
    got2 = host(lib.onnx_conv(dev(X), dev(Wt), None, pads, (2, 2), (1, 1), 1, residual=dev(R), act=1))
    assert rel_err(got2, ref2) <= REL_TOL
    # small integers: every partial sum exact, so the bits must agree whatever the order of the k pairs
    Xi = rng.integers(-4, 5, X.shape).astype(np.float32)
    Wi = rng.integers(-4, 5, Wt.shape).astype(np.float32)
    refi = oracle.conv(Xi, Wi, None, pads, (2, 2), (1, 1), 1)
    goti = host(lib.onnx_conv(dev(Xi), dev(Wi), None, pads, (2, 2), (1, 1), 1))
    assert np.array_equal(goti.astype(np.float64), refi)


@pytest.mark.parametrize("a,b,dH,dW,pads,st", [
    (1, 1, 1, 1, (1, 1, 1, 1), (1, 1)), (0, 2, 2, 1, (1, 0, 3, 2), (1, 1)), (2, 0, 1, 2, (0, 2, 1, 4), (2, 3)),
])
def test_conv_shifted_delta_kernel_bit_exact(lib, a, b, dH, dW, pads, st):
    """A filter that is 1 at one tap of the matching input channel copies (shifted, zero-filled,
    subsampled) input values: one non-zero product per output, so fp32 must reproduce it exactly."""
    announce("conv delta", a, b, dH, dW, pads, st)
    rng = np.random.default_rng(6)
    C = 32
    X = rng.standard_normal((3, C, 21, 17)).astype(np.float32)
    Wt = np.zeros((C, C, 3, 3), np.float32)
    for c in range(C):
        Wt[c, c, a, b] = 1.0
    ref = oracle.conv(X, Wt, None, pads, st, (dH, dW))
    got = host(lib.onnx_conv(dev(X), dev(Wt), None, pads, st, (dH, dW)))
    assert np.array_equal(got.astype(np.float64), ref)


def test_conv_small_integers_bit_exact(lib):
    announce("conv integer")
    rng = np.random.default_rng(8)
    X = rng.integers(-4, 5, (3, 48, 17, 19)).astype(np.float32)
    Wt = rng.integers(-4, 5, (72, 48, 3, 3)).astype(np.float32)
    Bv = rng.integers(-4, 5, (72,)).astype(np.float32)
    for pads, st, dl in [((1, 1, 1, 1), (1, 1), (1, 1)), ((0, 2, 1, 0), (2, 1), (1, 2))]:
        ref = oracle.conv(X, Wt, Bv, pads, st, dl)
        got = host(lib.onnx_conv(dev(X), dev(Wt), dev(Bv), pads, st, dl))
        assert np.array_equal(got.astype(np.float64), ref)


def test_conv_attribute_sweep_depthwise_full(lib):
    announce("conv depthwise full")
    c = workloads.attr_sweep_case("depthwise")
    for relu in (False, True):
        ref = oracle.conv(c["X"], c["W"], c["B"], c["pads"], c["strides"], c["dilations"], c["group"], relu=relu)
        got = host(lib.onnx_conv(dev(c["X"]), dev(c["W"]), dev(c["B"]), c["pads"], c["strides"],
                                 c["dilations"], c["group"], act=int(relu)))
        assert rel_err(got, ref) <= REL_TOL


def test_conv_attribute_sweep_dilated_full(lib):
    """8x512x28x28, 3x3, dilation 2, pad 2: all 8 images compared."""
    announce("conv dilated full")
    c = workloads.attr_sweep_case("dilated")
    ref, S = cached("dilated", lambda: oracle.conv(c["X"], c["W"], c["B"], c["pads"], c["strides"], c["dilations"],
                                                   c["group"], want_scale=True))
    got = host(lib.onnx_conv(dev(c["X"]), dev(c["W"]), dev(c["B"]), c["pads"], c["strides"], c["dilations"],
                             c["group"]))
    assert got.shape == (8, 512, 28, 28)
    assert rel_err(got, ref) <= REL_TOL
    assert within_rounding_bound(got, ref, S, 4608 + 1)


def test_conv_attribute_sweep_pointwise_full(lib):
    """32x1024x14x14 -> 256 channels, 1x1: all 32 images compared."""
    announce("conv pointwise full")
    c = workloads.attr_sweep_case("pointwise")
    ref = cached("pointwise", lambda: oracle.conv(c["X"], c["W"], c["B"], c["pads"], c["strides"], c["dilations"],
                                                  c["group"], relu=True))
    got = host(lib.onnx_conv(dev(c["X"]), dev(c["W"]), dev(c["B"]), c["pads"], c["strides"], c["dilations"],
                             c["group"], act=1))
    assert rel_err(got, ref) <= REL_TOL


def test_nan_and_inf_propagate_alike_on_every_conv_path(lib):
    """A NaN or an infinity in the input reaches the output the same way whichever kernel the shape
    selects: without Relu the affected outputs are NaN / inf, with Relu a NaN becomes 0 (the
    v > 0 ? v : 0 of the definition) and +inf stays +inf."""
    announce("nan/inf propagation")
    rng = np.random.default_rng(99)
    shapes = [
        ((2, 16, 12, 12), (32, 16, 3, 3), (1, 1, 1, 1), 1),      # LDS-patch kernel
        ((2, 16, 12, 12), (32, 16, 1, 1), (0, 0, 0, 0), 1),      # contraction kernel
        ((2, 6, 12, 12), (32, 6, 5, 5), (2, 2, 2, 2), 1),        # gather loader
        ((2, 8, 12, 12), (8, 1, 3, 3), (1, 1, 1, 1), 8),         # row-strip (depthwise)
        ((2, 8, 12, 12), (8, 1, 5, 5), (2, 2, 2, 2), 8),         # direct
        ((2, 3, 20, 20), (32, 3, 7, 7), (3, 3, 3, 3), 1),        # gather loader, 7x7 stride 2
        ((256, 3, 20, 20), (32, 3, 7, 7), (3, 3, 3, 3), 1),      # filters resident in registers (stride 2)
    ]
    for xs, ws_, pads, g in shapes:
        X = rng.uniform(0.5, 1, xs).astype(np.float32)
        Wt = rng.uniform(0.5, 1, ws_).astype(np.float32)
        X[0, 0, 5, 5] = np.nan
        X[1, 1, 6, 6] = np.inf
        for relu in (False, True):
            st = (2, 2) if ws_[2] == 7 else (1, 1)
            ref = oracle.conv(X, Wt, None, pads, st, (1, 1), g, relu=relu)
            got = host(lib.onnx_conv(dev(X), dev(Wt), None, pads, st, (1, 1), g, act=int(relu)))
            assert np.array_equal(np.isnan(got), np.isnan(ref)), (xs, ws_, relu)
            assert np.array_equal(np.isinf(got), np.isinf(ref)), (xs, ws_, relu)
            fin = np.isfinite(ref)
            assert rel_err(np.where(fin, got, 0), np.where(fin, ref, 0)) <= REL_TOL
    # Gemm (contraction epilogue, every split configuration of the fixture)
    A = rng.uniform(0.5, 1, (70, 300)).astype(np.float32)
    B = rng.uniform(0.5, 1, (300, 90)).astype(np.float32)
    A[3, 7] = np.nan
    A[9, 1] = -np.inf
    for relu in (False, True):
        ref = oracle.gemm(A, B, None, 1.0, 1.0, 0, 0, relu=relu)
        got = host(lib.onnx_gemm(dev(A), dev(B), act=int(relu)))
        assert np.array_equal(np.isnan(got), np.isnan(ref)) and np.array_equal(np.isinf(got), np.isinf(ref)), relu


# ------------------------------------------------------------------------------ pools

POOL_CASES = [
    (2, 3, 9, 8, (3, 3), (1, 1, 1, 1), (2, 2), (1, 1), 0),
    (1, 2, 10, 7, (2, 3), (0, 1, 0, 1), (2, 1), (1, 1), 0),
    (2, 2, 11, 11, (3, 3), (1, 1, 1, 1), (2, 2), (1, 1), 1),
    (1, 3, 12, 9, (3, 2), (0, 0, 0, 0), (3, 2), (2, 2), 0),
    (1, 1, 7, 7, (2, 2), (0, 0, 0, 0), (2, 2), (1, 1), 1),
    (2, 5, 13, 10, (3, 2), (2, 0, 1, 1), (1, 2), (1, 1), 0),
    (3, 64, 56, 56, (3, 3), (1, 1, 1, 1), (2, 2), (1, 1), 0),
    # vertical stride 2 (row-strip kernel): several column chunks, ragged strips, ceil_mode, horizontal stride / dilation
    (2, 3, 37, 300, (3, 3), (1, 1, 1, 1), (2, 2), (1, 1), 0),
    (1, 2, 30, 131, (2, 2), (0, 0, 0, 0), (2, 2), (1, 1), 1),
    (2, 2, 19, 90, (3, 3), (1, 0, 0, 1), (2, 1), (1, 2), 1),
    (1, 3, 9, 70, (2, 2), (1, 1, 1, 1), (2, 3), (1, 1), 0),
    (2, 4, 3, 3, (3, 3), (1, 1, 1, 1), (2, 2), (1, 1), 0),
    # even width, horizontal stride 2, left pad = kernel - 2: the 8-byte paired loads
    (2, 3, 12, 20, (2, 2), (0, 0, 0, 0), (2, 2), (1, 1), 0),
    (1, 2, 16, 24, (3, 3), (1, 1, 0, 2), (2, 2), (1, 1), 1),
    (2, 2, 9, 128, (3, 3), (0, 1, 1, 1), (2, 2), (1, 1), 0),
    (1, 2, 11, 130, (3, 3), (1, 1, 1, 1), (2, 2), (1, 1), 0),        # 65 output columns: two chunks, plain loads
    (2, 3, 9, 10, (2, 2), (0, 0, 0, 0), (1, 1), (1, 1), 0),          # 2x2 window, stride 1: the plane-strip kernel
]


@pytest.mark.parametrize("case", POOL_CASES)
def test_maxpool_bit_exact_with_indices(lib, case):
    announce("maxpool", case)
    N, C, H, W, k, pads, st, dl, ceil = case
    rng = np.random.default_rng(31)
    X = rng.integers(-3, 4, (N, C, H, W)).astype(np.float32)          # many ties
    X += (rng.random((N, C, H, W)) < 0.5).astype(np.float32) * 0.5
    ref, iref = oracle.maxpool(X, k, pads, st, dl, ceil)
    got, igot = lib.onnx_maxpool(dev(X), k, pads, st, dl, ceil, want_indices=True)
    got, igot = host(got), host(igot)
    assert np.array_equal(got, ref)
    assert np.array_equal(igot, iref)
    only = host(lib.onnx_maxpool(dev(X), k, pads, st, dl, ceil))
    assert np.array_equal(only, ref)


def test_maxpool_resnet_stem_shape_values_and_indices(lib):
    """32x64x112x112, 3x3 / stride 2 / pad 1 (the pool behind ResNet-50's stem at batch 32, the
    shape the benchmark times): every value and every int64 index, bit for bit."""
    announce("maxpool 32x64x112x112")
    rng = np.random.default_rng(41)
    X = rng.integers(-6, 7, (32, 64, 112, 112)).astype(np.float32)      # ties in most windows
    X += (rng.random(X.shape) < 0.3).astype(np.float32) * 0.25
    ref, iref = cached("maxpool_stem", lambda: oracle.maxpool(X, (3, 3), (1, 1, 1, 1), (2, 2), (1, 1), 0))
    got, igot = lib.onnx_maxpool(dev(X), (3, 3), (1, 1, 1, 1), (2, 2), (1, 1), 0, want_indices=True)
    assert np.array_equal(host(got), ref)
    assert np.array_equal(host(igot), iref)
    assert np.array_equal(host(lib.onnx_maxpool(dev(X), (3, 3), (1, 1, 1, 1), (2, 2))), ref)


@pytest.mark.parametrize("case", POOL_CASES)
@pytest.mark.parametrize("cip", [0, 1])
def test_avgpool_matches_oracle(lib, case, cip):
    announce("avgpool", case, cip)
    N, C, H, W, k, pads, st, dl, ceil = case
    rng = np.random.default_rng(34)
    X = rng.standard_normal((N, C, H, W)).astype(np.float32)
    ref = oracle.avgpool(X, k, pads, st, ceil, cip)
    got = host(lib.onnx_avgpool(dev(X), k, pads, st, ceil, cip))
    assert rel_err(got, ref) <= REL_TOL


@pytest.mark.parametrize("shape", [(2, 5, 7, 7), (3, 130, 1, 1), (1, 3, 20, 33), (32, 2048, 7, 7)])
def test_global_avgpool_matches_oracle(lib, shape):
    announce("global avgpool", shape)
    rng = np.random.default_rng(35)
    X = rng.standard_normal(shape).astype(np.float32)
    ref = oracle.avgpool(X, None)
    got = host(lib.onnx_avgpool(dev(X), None))
    assert got.shape == ref.shape
    assert rel_err(got, ref) <= REL_TOL


def test_split_k_shapes_repeatable(lib, workspace):
    """Few output tiles and a long K: with a workspace the K range is split, partial tiles go
    through the workspace and a second kernel adds them in split order.  Each case runs three
    times: the result must be bit-identical from run to run."""
    announce("split-k", workspace)
    rng = np.random.default_rng(77)
    for (M, N, K) in [(64, 64, 4096), (100, 130, 2500), (1, 1000, 2048), (32, 1000, 2048), (256, 49, 4608)]:
        A = rng.uniform(-1, 1, (M, K)).astype(np.float32)
        B = rng.uniform(-1, 1, (N, K)).astype(np.float32)
        C = rng.uniform(-1, 1, (1, N)).astype(np.float32)
        ref, S = oracle.gemm(A, B, C, 1.0, 1.0, 0, 1, relu=False, want_scale=True)
        a, b, c = dev(A), dev(B), dev(C)
        outs = [host(lib.onnx_gemm(a, b, c, 1.0, 1.0, 0, 1)) for _ in range(3)]
        assert rel_err(outs[0], ref) <= REL_TOL
        assert within_rounding_bound(outs[0], ref, S, K + 2)
        assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])
    X = rng.uniform(-1, 1, (1, 512, 7, 7)).astype(np.float32)
    Wt = rng.uniform(-1, 1, (512, 512, 3, 3)).astype(np.float32)
    Bv = rng.uniform(-1, 1, (512,)).astype(np.float32)
    R = rng.uniform(-1, 1, (1, 512, 7, 7)).astype(np.float32)
    ref = oracle.conv(X, Wt, Bv, (1, 1, 1, 1), residual=R, relu=True)
    x, w, bv, r = dev(X), dev(Wt), dev(Bv), dev(R)
    outs = [host(lib.onnx_conv(x, w, bv, (1, 1, 1, 1), residual=r, act=1)) for _ in range(3)]
    assert rel_err(outs[0], ref) <= REL_TOL
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])
    X = rng.uniform(-1, 1, (2, 1024, 14, 14)).astype(np.float32)
    Wt = rng.uniform(-1, 1, (256, 1024, 1, 1)).astype(np.float32)
    ref = oracle.conv(X, Wt, None)
    assert rel_err(host(lib.onnx_conv(dev(X), dev(Wt), None)), ref) <= REL_TOL


def test_tail_split_shapes_repeatable(lib, workspace):
    """Slightly more than a multiple of 256 output tiles: with a workspace the surplus tiles are
    shared by several workgroups each (their K range cut into shares) inside the same launch and
    finished by a second kernel; the rest of the tiles is computed as usual.  Results must match
    the oracle everywhere (whole tiles, shared tiles, ragged edges) and repeat bit for bit."""
    announce("tail-split", workspace)
    rng = np.random.default_rng(78)
    # 64x64 tiles: 17x16 = 272 (16 surplus), 18x16 with ragged edges = 288 (32 surplus), 25x31 = 775 (7 surplus)
    for (M, N, K, tA, tB) in [(1088, 1024, 256, 0, 1), (1100, 1000, 300, 0, 0), (1600, 1984, 128, 1, 1)]:
        A = rng.uniform(-1, 1, (K, M) if tA else (M, K)).astype(np.float32)
        B = rng.uniform(-1, 1, (N, K) if tB else (K, N)).astype(np.float32)
        C = rng.uniform(-1, 1, (1, N)).astype(np.float32)
        ref, S = oracle.gemm(A, B, C, 1.0, 1.0, tA, tB, relu=False, want_scale=True)
        a, b, c = dev(A), dev(B), dev(C)
        outs = [host(lib.onnx_gemm(a, b, c, 1.0, 1.0, tA, tB)) for _ in range(3)]
        assert rel_err(outs[0], ref) <= REL_TOL
        assert within_rounding_bound(outs[0], ref, S, K + 2)
        assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])
    # 3x3 convolution through the LDS-patch kernel: 2 x 400 = 800 tiles of 64x64 (32 surplus), bias + residual + Relu
    X = rng.uniform(-1, 1, (32, 64, 28, 29)).astype(np.float32)
    Wt = rng.uniform(-1, 1, (128, 64, 3, 3)).astype(np.float32)
    Bv = rng.uniform(-1, 1, (128,)).astype(np.float32)
    R = rng.uniform(-1, 1, (32, 128, 28, 29)).astype(np.float32)
    ref = oracle.conv(X, Wt, Bv, (1, 1, 1, 1), residual=R, relu=True)
    x, w_, bv, r = dev(X), dev(Wt), dev(Bv), dev(R)
    outs = [host(lib.onnx_conv(x, w_, bv, (1, 1, 1, 1), residual=r, act=1)) for _ in range(2)]
    assert rel_err(outs[0], ref) <= REL_TOL
    assert np.array_equal(outs[0], outs[1])
    # 1x1 convolution (row-contiguous loader): 4 x 196 = 784 tiles
    X = rng.uniform(-1, 1, (16, 128, 28, 28)).astype(np.float32)
    Wt = rng.uniform(-1, 1, (256, 128, 1, 1)).astype(np.float32)
    ref = oracle.conv(X, Wt, None)
    assert rel_err(host(lib.onnx_conv(dev(X), dev(Wt), None)), ref) <= REL_TOL


# ------------------------------------------------------------------------------ degenerate sizes and errors

def test_zero_sized_outputs_return_ok(lib):
    announce("zero sized")
    z = torch.empty((0, 8), dtype=torch.float32, device="cuda")
    b = torch.ones((8, 5), dtype=torch.float32, device="cuda")
    assert tuple(lib.onnx_gemm(z, b).shape) == (0, 5)
    assert tuple(lib.onnx_matmul(z, b).shape) == (0, 5)
    x = torch.empty((0, 3, 8, 8), dtype=torch.float32, device="cuda")
    w = torch.ones((4, 3, 3, 3), dtype=torch.float32, device="cuda")
    assert tuple(lib.onnx_conv(x, w).shape) == (0, 4, 6, 6)
    assert tuple(lib.onnx_maxpool(x, (2, 2)).shape) == (0, 3, 7, 7)
    assert tuple(lib.onnx_avgpool(x, None).shape) == (0, 3, 1, 1)
    # K = 0: an empty sum plus the bias
    a = torch.empty((3, 0), dtype=torch.float32, device="cuda")
    bb = torch.empty((0, 4), dtype=torch.float32, device="cuda")
    c = torch.full((1, 4), 2.5, dtype=torch.float32, device="cuda")
    assert np.array_equal(host(lib.onnx_gemm(a, bb, c)), np.full((3, 4), 2.5, np.float32))


def test_errors_write_nothing(lib):
    announce("errors")
    a = torch.ones((4, 4), dtype=torch.float32, device="cuda")
    y = torch.full((4, 4), 7.0, dtype=torch.float32, device="cuda")
    with pytest.raises(lib.OnnxHipError) as e:
        lib.onnx_gemm(a, a, out=a)                                   # output aliases an input
    assert e.value.status == 6
    with pytest.raises(lib.OnnxHipError) as e:
        lib.onnx_gemm(a, torch.ones((5, 4), dtype=torch.float32, device="cuda"), out=y)
    assert e.value.status == 3
    assert np.array_equal(host(y), np.full((4, 4), 7.0, np.float32))


# ------------------------------------------------------------------------------ model chains

def _run_chain(lib, model, workspace="workspace"):
    """The runner sets its own workspace at the start of a run: none or 64 MiB, following the fixture."""
    from paper_2008_08272_amd.runner import GraphRunner
    r = GraphRunner(model, workspace_bytes=(64 << 20) if workspace == "workspace" else 0, keep_intermediates=True)
    out = r.run()
    torch.cuda.synchronize()
    return r, out.cpu().numpy()


def test_small_cnn_chain(lib, workspace):
    announce("small cnn chain")
    from oracle import chain
    m = workloads.small_cnn()
    env, exact = chain.run(m)
    r, got = _run_chain(lib, m, workspace)
    assert rel_err(got, exact["logits"]) <= REL_TOL
    for name in ("c1", "p1", "c2", "p2"):
        assert rel_err(r.t[name].cpu().numpy(), exact[name]) <= REL_TOL, name


def test_resnet50_batch1_chain(lib, workspace):
    announce("resnet50 b1 chain")
    from oracle import chain
    m = workloads.resnet50(1)
    env, exact = chain.run(m)
    r, got = _run_chain(lib, m, workspace)
    worst = 0.0
    for nd in m["graph"]:
        if nd["op"] == "reshape":
            continue
        e = rel_err(r.t[nd["y"]].cpu().numpy(), exact[nd["y"]])
        worst = max(worst, e)
        assert e <= REL_TOL, (nd["y"], e)
    print("resnet50 b1 worst layer error", worst, flush=True)
    assert rel_err(got, exact["logits"]) <= REL_TOL


def test_resnet50_batch1_graph_replay(lib):
    """The batch-1 chain captured into a HIP graph: every replay, with eager work and
    synchronisation in between, must reproduce the eager result bit for bit."""
    announce("resnet50 b1 graph")
    from paper_2008_08272_amd.runner import GraphRunner
    m = workloads.resnet50(1)
    r = GraphRunner(m)
    eager = r.run().clone()
    torch.cuda.synchronize()
    r.capture()
    rng = np.random.default_rng(5)
    for i in range(4):
        r.output.zero_()
        junk = lib.onnx_gemm(dev(rng.uniform(-1, 1, (70, 90)).astype(np.float32)),
                             dev(rng.uniform(-1, 1, (90, 50)).astype(np.float32)))
        torch.cuda.synchronize()
        out = r.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), i
        del junk
    # a new input through the same graph
    x2 = rng.standard_normal(m["inputs"]["x"].shape).astype(np.float32)
    r.set_input("x", x2)
    got = host(r.replay())
    from oracle import chain
    m2 = dict(m)
    m2["inputs"] = {"x": x2}
    _, exact = chain.run(m2, keep=())
    assert rel_err(got, exact["logits"]) <= REL_TOL


def test_resnet50_batch32_chain_every_image_every_layer(lib, workspace):
    """The batch-32 launch shapes the benchmark times.  The oracle runs the same graph image by
    image (an image's activations depend on that image only) and every activation of every one of
    the 32 images is compared, layer by layer."""
    announce("resnet50 b32 chain")
    from oracle import chain
    m = workloads.resnet50(32)
    r, got = _run_chain(lib, m, workspace)
    assert got.shape == (32, 1000)
    layers = [nd["y"] for nd in m["graph"] if nd["op"] != "reshape"]
    acts = {name: r.t[name].cpu().numpy() for name in layers}
    worst = 0.0
    for n in range(32):
        def one_image(n=n):
            sub = dict(m)
            sub["inputs"] = {"x": m["inputs"]["x"][n:n + 1]}
            sub["graph"] = [dict(nd, shape=(1, 2048)) if nd["op"] == "reshape" else nd for nd in m["graph"]]
            return {k: np.asarray(v, dtype=np.float32) for k, v in chain.run(sub)[1].items()}
        # kept for the second workspace configuration as fp32 (2^-24 relative: far below the tolerance)
        exact = cached(("resnet50_b32", n), one_image)
        for name in layers:
            e = rel_err(acts[name][n:n + 1], exact[name])
            worst = max(worst, e)
            assert e <= REL_TOL, (n, name, e)
    print("resnet50 b32 worst layer error", worst, flush=True)


# ------------------------------------------------------------------------------ graph passes

def test_unfused_graphs_through_the_passes(lib, workspace):
    """Operator-by-operator graphs (BatchNormalization, Relu, Add, Identity, MatMul + Add as nodes
    of their own) go through the graph passes and then through the runner; the reference is the
    oracle evaluating the ORIGINAL graph by the operators' definitions."""
    announce("passes + runner")
    from oracle import chain
    from paper_2008_08272_amd import passes
    from paper_2008_08272_amd.runner import GraphRunner
    for raw in (workloads.small_cnn_unfused(), workloads.resnet50_unfused(2, image=96)):
        with pytest.raises(NotImplementedError):
            GraphRunner(raw)                     # no kernel for a bare Relu / BatchNorm: fails loudly
        opt = passes.optimize(raw)
        _, exact = chain.run(raw)
        r, got = _run_chain(lib, opt, workspace)
        assert got.shape == exact[raw["output"]].shape
        assert rel_err(got, exact[raw["output"]]) <= REL_TOL, raw["name"]
        # every intermediate tensor that survives the rewrite matches the original graph's
        worst = 0.0
        for nd in opt["graph"]:
            if nd["op"] != "reshape" and nd["y"] in exact:
                worst = max(worst, rel_err(r.t[nd["y"]].cpu().numpy(), exact[nd["y"]]))
        assert worst <= REL_TOL


def test_constant_propagation_graph_on_the_gpu(lib, workspace):
    """Chained Adds of constants (the paper's normalisation rules, Section 3.4): the rewritten graph
    runs on the GPU, the reference is the oracle on the graph as written."""
    announce("constant propagation + runner")
    from oracle import chain
    from paper_2008_08272_amd import passes
    raw = workloads.constant_adds()
    _, exact = chain.run(raw)
    opt = passes.optimize(raw)
    assert sum(nd["op"] == "add" for nd in opt["graph"]) == 4
    r, got = _run_chain(lib, opt, workspace)
    assert rel_err(got, exact["out"]) <= REL_TOL
    _, got_raw = _run_chain(lib, raw, workspace)           # the unrewritten graph runs too, operator by operator
    assert rel_err(got_raw, exact["out"]) <= REL_TOL


# ------------------------------------------------------------------------------ seeded random sweeps

def _random_conv_case(rng):
    kH, kW = [(1, 1), (3, 3), (3, 3), (3, 3), (5, 5), (2, 3), (7, 7), (1, 3)][int(rng.integers(0, 8))]
    group = int(rng.choice([1, 1, 1, 2, 4]))
    cg = int(rng.choice([1, 3, 4, 8, 12, 16, 32]))
    mg = int(rng.choice([1, 4, 16, 24, 64, 80]))
    C, M = cg * group, mg * group
    sH, sW = int(rng.integers(1, 4)), int(rng.integers(1, 4))
    dH, dW = int(rng.integers(1, 3)), int(rng.integers(1, 3))
    pads = tuple(int(rng.integers(0, 3)) for _ in range(4))
    eh, ew = (kH - 1) * dH + 1, (kW - 1) * dW + 1
    H = int(rng.integers(max(1, eh - pads[0] - pads[2]), 40))
    W = int(rng.integers(max(1, ew - pads[1] - pads[3]), 40))
    N = int(rng.integers(1, 5))
    return (N, C, H, W, M, kH, kW, pads, (sH, sW), (dH, dW), group)


def test_conv_random_attribute_sweep(lib):
    """120 seeded random convolutions over kernel sizes, groups, channel counts, pads, strides and
    dilations: whatever path the selector takes (matrix cores with the LDS patch, the gather or
    the row-contiguous loaders, row-strip, plane or direct kernels), the result must match."""
    rng = np.random.default_rng(20260)
    for it in range(120):
        case = _random_conv_case(rng)
        N, C, H, W, M, kH, kW, pads, st, dl, g = case
        announce("conv sweep", it, case)
        X = rng.uniform(-1, 1, (N, C, H, W)).astype(np.float32)
        Wt = rng.uniform(-1, 1, (M, C // g, kH, kW)).astype(np.float32)
        Bv = rng.uniform(-1, 1, (M,)).astype(np.float32) if it % 3 else None
        relu = bool(it % 2)
        ref = oracle.conv(X, Wt, Bv, pads, st, dl, g, relu=relu)
        R = rng.uniform(-1, 1, ref.shape).astype(np.float32) if it % 4 == 0 else None
        if R is not None:
            ref = oracle.conv(X, Wt, Bv, pads, st, dl, g, residual=R, relu=relu)
        got = host(lib.onnx_conv(dev(X), dev(Wt), dev(Bv), pads, st, dl, g, residual=dev(R), act=int(relu)))
        assert got.shape == ref.shape, case
        assert rel_err(got, ref) <= REL_TOL, case


def test_gemm_matmul_random_sweep(lib):
    rng = np.random.default_rng(20261)
    for it in range(60):
        M, N, K = (int(rng.integers(1, 400)) for _ in range(3))
        if it % 5 == 0:
            K = int(rng.integers(400, 3000))
        tA, tB = int(rng.integers(0, 2)), int(rng.integers(0, 2))
        announce("gemm sweep", it, M, N, K, tA, tB)
        A = rng.uniform(-1, 1, (K, M) if tA else (M, K)).astype(np.float32)
        B = rng.uniform(-1, 1, (N, K) if tB else (K, N)).astype(np.float32)
        cshape = [(1, N), (M, 1), (M, N), (N,), None][it % 5]
        C = rng.uniform(-1, 1, cshape).astype(np.float32) if cshape else None
        alpha, beta = float(np.float32(rng.uniform(-2, 2))), float(np.float32(rng.uniform(-2, 2)))
        ref, S = oracle.gemm(A, B, C, alpha, beta, tA, tB, relu=bool(it % 2), want_scale=True)
        got = host(lib.onnx_gemm(dev(A), dev(B), dev(C), alpha, beta, tA, tB, act=it % 2))
        assert rel_err(got, ref) <= REL_TOL
        assert within_rounding_bound(got, ref, S, K + 2)
    for it in range(20):
        batch = tuple(int(rng.integers(1, 4)) for _ in range(int(rng.integers(0, 3))))
        m, n, k = (int(rng.integers(1, 90)) for _ in range(3))
        sa = tuple(b if rng.random() < 0.7 else 1 for b in batch) + (m, k)
        sb = tuple(b if rng.random() < 0.7 else 1 for b in batch)[int(rng.integers(0, len(batch) + 1)):] + (k, n)
        announce("matmul sweep", it, sa, sb)
        A = rng.uniform(-1, 1, sa).astype(np.float32)
        B = rng.uniform(-1, 1, sb).astype(np.float32)
        ref = oracle.matmul(A, B)
        got = host(lib.onnx_matmul(dev(A), dev(B)))
        assert got.shape == ref.shape
        assert rel_err(got, ref) <= REL_TOL


def test_pool_random_sweep(lib):
    rng = np.random.default_rng(20262)
    for it in range(80):
        kH, kW = int(rng.integers(1, 5)), int(rng.integers(1, 5))
        sH, sW = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        dH, dW = int(rng.integers(1, 3)), int(rng.integers(1, 3))
        pads = (int(rng.integers(0, kH)), int(rng.integers(0, kW)), int(rng.integers(0, kH)), int(rng.integers(0, kW)))
        ceil = int(rng.integers(0, 2))
        H = int(rng.integers((kH - 1) * dH + 1, 50))
        W = int(rng.integers((kW - 1) * dW + 1, 140))
        N, C = int(rng.integers(1, 3)), int(rng.integers(1, 5))
        announce("pool sweep", it, (N, C, H, W), (kH, kW), pads, (sH, sW), (dH, dW), ceil)
        X = rng.integers(-4, 5, (N, C, H, W)).astype(np.float32) + (rng.random((N, C, H, W)) < 0.5) * np.float32(0.5)
        X = X.astype(np.float32)
        ref, iref = oracle.maxpool(X, (kH, kW), pads, (sH, sW), (dH, dW), ceil)
        got, igot = lib.onnx_maxpool(dev(X), (kH, kW), pads, (sH, sW), (dH, dW), ceil, want_indices=True)
        assert np.array_equal(host(got), ref)
        assert np.array_equal(host(igot), iref)
        for cip in (0, 1):
            ra = oracle.avgpool(X, (kH, kW), pads, (sH, sW), ceil, cip)
            ga = host(lib.onnx_avgpool(dev(X), (kH, kW), pads, (sH, sW), ceil, cip))
            assert rel_err(ga, ra) <= REL_TOL


# ------------------------------------------------------------------------------ every kernel instance

def _offset_dev(a, misalign):
    """The array on the GPU; with `misalign` its first element sits 4 bytes past a 16-byte boundary
    (a view into a larger buffer), which rules out 16-byte loads of that operand."""
    if not misalign:
        return dev(a)
    buf = torch.empty(a.size + 1, dtype=torch.float32, device="cuda")
    view = buf[1:].view(a.shape)
    view.copy_(torch.from_numpy(np.ascontiguousarray(a)))
    assert view.data_ptr() % 16 == 4
    return view


# tile class -> (M, N, K) that makes the selector take it, and the instance it names
GEMM_TILE_CLASSES = {
    "64x64x16": ((132, 200, 72), "64x64x16 waves 2x2x1"),
    "64x64x32": ((1500, 1504, 512), "64x64x32 waves 2x2x1"),
    "64x64x32 sliced": ((800, 900, 300), "64x64x32 waves 2x2x2"),
    "32x32x64 sliced": ((200, 152, 300), "32x32x64 waves 1x1x4"),
    "128x128x16": ((2048, 2048, 512), "128x128x16 waves 4x4x1"),
    "256x256x16": ((4096, 4096, 40), "256x256x16 waves 4x4x1"),
}


@pytest.mark.parametrize("loads", ["16B/16B", "16B/4B", "4B/4B"])
@pytest.mark.parametrize("transA,transB", [(0, 1), (0, 0), (1, 1), (1, 0)])
@pytest.mark.parametrize("tile", list(GEMM_TILE_CLASSES))
def test_every_gemm_instance(lib, tile, transA, transB, loads):
    """One case per compiled instance of the contraction kernel that Gemm can reach: tile shape x
    operand layouts x load widths.  The launch record names the instance that ran; the whole
    output is compared with the oracle."""
    (M, N, K), inst = GEMM_TILE_CLASSES[tile]
    announce("gemm instance", tile, transA, transB, loads)
    rng = np.random.default_rng([M, N, K, transA, transB])
    A = rng.uniform(-1, 1, (K, M) if transA else (M, K)).astype(np.float32)
    B = rng.uniform(-1, 1, (N, K) if transB else (K, N)).astype(np.float32)
    C = rng.uniform(-1, 1, (1, N)).astype(np.float32)
    ref, S = cached(("gemm_inst", tile, transA, transB),
                    lambda: oracle.gemm(A, B, C, 1.0, 1.0, transA, transB, want_scale=True))
    a = _offset_dev(A, loads == "4B/4B")
    b = _offset_dev(B, loads != "16B/16B")
    got = host(lib.onnx_gemm(a, b, dev(C), 1.0, 1.0, transA, transB))
    av, bv = {"16B/16B": (4, 4), "16B/4B": (4, 1), "4B/4B": (1, 1)}[loads]
    want = "contraction %s A=%s/%d B=%s/%d " % (inst, "RC" if transA else "KC", av, "KC" if transB else "RC", bv)
    assert lib.onnx_last_launch().startswith(want), (lib.onnx_last_launch(), want)
    assert rel_err(got, ref) <= REL_TOL
    assert within_rounding_bound(got, ref, S, K + 2)


CONV_INSTANCE_CASES = [
    # name, X shape, W shape, pads, strides, expected instance prefix
    ("im2col 64x64x16 16B", (1, 8, 14, 14), (16, 8, 5, 5), (2, 2, 2, 2), (1, 1), "64x64x16 waves 2x2x1 A=KC/4 B=IM2COL/1"),
    ("im2col 64x64x16 4B", (2, 3, 37, 41), (64, 3, 5, 5), (2, 2, 2, 2), (2, 2), "64x64x16 waves 2x2x1 A=KC/1 B=IM2COL/1"),
    ("im2col 64x64x32 16B", (16, 24, 48, 48), (64, 24, 5, 5), (2, 2, 2, 2), (1, 1), "64x64x32 waves 2x2x1 A=KC/4 B=IM2COL/1"),
    ("im2col 64x64x32 4B", (16, 25, 48, 48), (64, 25, 5, 5), (2, 2, 2, 2), (1, 1), "64x64x32 waves 2x2x1 A=KC/1 B=IM2COL/1"),
    ("im2col sliced 16B", (2, 24, 20, 20), (64, 24, 5, 5), (2, 2, 2, 2), (1, 1), "64x64x32 waves 2x2x2 A=KC/4 B=IM2COL/1"),
    ("im2col sliced 4B", (2, 25, 20, 20), (64, 25, 5, 5), (2, 2, 2, 2), (1, 1), "64x64x32 waves 2x2x2 A=KC/1 B=IM2COL/1"),
    ("im2col 128x128x16 16B", (2, 24, 64, 64), (512, 24, 5, 5), (2, 2, 2, 2), (1, 1), "128x128x16 waves 4x4x1 A=KC/4 B=IM2COL/1"),
    ("im2col 128x128x16 4B", (2, 21, 64, 64), (512, 21, 5, 5), (2, 2, 2, 2), (1, 1), "128x128x16 waves 4x4x1 A=KC/1 B=IM2COL/1"),
    ("im2col 256x256x16 16B", (8, 4, 64, 64), (512, 4, 5, 5), (2, 2, 2, 2), (1, 1), "256x256x16 waves 4x4x1 A=KC/4 B=IM2COL/1"),
    ("im2col 256x256x16 4B", (8, 6, 64, 64), (512, 6, 3, 3), (1, 1, 1, 1), (1, 1), "256x256x16 waves 4x4x1 A=KC/1 B=IM2COL/1"),
    ("rcs 64x64x16 16B", (2, 64, 12, 12), (96, 64, 1, 1), (0, 0, 0, 0), (2, 2), "64x64x16 waves 2x2x1 A=KC/4 B=RCS/1"),
    ("rcs 64x64x16 4B", (2, 18, 13, 11), (40, 18, 1, 1), (0, 0, 0, 0), (3, 2), "64x64x16 waves 2x2x1 A=KC/1 B=RCS/1"),
    ("rcs 64x64x32 16B", (9, 512, 64, 64), (256, 512, 1, 1), (0, 0, 0, 0), (2, 2), "64x64x32 waves 2x2x1 A=KC/4 B=RCS/1"),
    ("rcs 64x64x32 4B", (9, 514, 64, 64), (256, 514, 1, 1), (0, 0, 0, 0), (2, 2), "64x64x32 waves 2x2x1 A=KC/1 B=RCS/1"),
    ("rcs sliced 16B", (8, 512, 56, 56), (128, 512, 1, 1), (0, 0, 0, 0), (2, 2), "64x64x32 waves 2x2x2 A=KC/4 B=RCS/1"),
    ("rcs sliced 4B", (8, 510, 56, 56), (128, 510, 1, 1), (0, 0, 0, 0), (2, 2), "64x64x32 waves 2x2x2 A=KC/1 B=RCS/1"),
    ("rcs 32x32x64 sliced 16B", (2, 512, 14, 14), (128, 512, 1, 1), (0, 0, 0, 0), (2, 2), "32x32x64 waves 1x1x4 A=KC/4 B=RCS/1"),
    ("rcs 32x32x64 sliced 4B", (2, 510, 14, 14), (128, 510, 1, 1), (0, 0, 0, 0), (2, 2), "32x32x64 waves 1x1x4 A=KC/1 B=RCS/1"),
    ("rcs 128x128x16 16B", (2, 512, 128, 128), (512, 512, 1, 1), (0, 0, 0, 0), (2, 2), "128x128x16 waves 4x4x1 A=KC/4 B=RCS/1"),
    ("rcs 128x128x16 4B", (2, 514, 128, 128), (512, 514, 1, 1), (0, 0, 0, 0), (2, 2), "128x128x16 waves 4x4x1 A=KC/1 B=RCS/1"),
    ("rcs 256x256x16 16B", (8, 16, 128, 128), (512, 16, 1, 1), (0, 0, 0, 0), (2, 2), "256x256x16 waves 4x4x1 A=KC/4 B=RCS/1"),
    ("rcs 256x256x16 4B", (8, 18, 128, 128), (512, 18, 1, 1), (0, 0, 0, 0), (2, 2), "256x256x16 waves 4x4x1 A=KC/1 B=RCS/1"),
    # pointwise convolutions: the row-contiguous loader with images as column blocks
    ("pointwise 16B/16B", (2, 64, 12, 12), (96, 64, 1, 1), (0, 0, 0, 0), (1, 1), "64x64x16 waves 2x2x1 A=KC/4 B=RC/4"),
    ("pointwise 16B/4B (P = 49)", (32, 512, 7, 7), (2048, 512, 1, 1), (0, 0, 0, 0), (1, 1), "64x64x32 waves 2x2x1 A=KC/4 B=RC/1"),
    ("pointwise 32x32x64 sliced (P = 49)", (1, 512, 7, 7), (2048, 512, 1, 1), (0, 0, 0, 0), (1, 1), "32x32x64 waves 1x1x4 A=KC/4 B=RC/1"),
    ("pointwise 32x32x64 sliced", (1, 256, 14, 14), (1024, 256, 1, 1), (0, 0, 0, 0), (1, 1), "32x32x64 waves 1x1x4 A=KC/4 B=RC/4"),
    ("pointwise 128x128x16", (8, 512, 32, 32), (512, 512, 1, 1), (0, 0, 0, 0), (1, 1), "128x128x16 waves 4x4x1 A=KC/4 B=RC/4"),
    ("pointwise 256x256x16", (32, 64, 32, 32), (512, 64, 1, 1), (0, 0, 0, 0), (1, 1), "256x256x16 waves 4x4x1 A=KC/4 B=RC/4"),
]


CONV_WINDOW_INSTANCE_CASES = [
    # name, X shape, output channels, pad = dilation, stride, expected instance, and what the split looks like with a workspace
    ("64x64 2 passes", (30, 16, 16, 4), 64, 1, 1, "64x64x36 waves 2x2x1 A=KC/4 B=IM2COL/1 npb=2", None),
    ("128x128 2 passes", (500, 16, 8, 8), 128, 1, 1, "128x128x36 waves 4x2x1 A=KC/4 B=IM2COL/1 npb=2", None),
    ("128x128 3 passes", (500, 16, 8, 8), 128, 2, 1, "128x128x36 waves 4x2x1 A=KC/4 B=IM2COL/1 npb=3", None),
    ("128x128 4 passes", (500, 16, 8, 8), 128, 3, 1, "128x128x36 waves 4x2x1 A=KC/4 B=IM2COL/1 npb=4", None),
    ("128x128 5 passes", (500, 16, 16, 16), 128, 1, 2, "128x128x36 waves 4x2x1 A=KC/4 B=IM2COL/1 npb=5", None),
    ("128x128 6 passes", (2000, 16, 8, 8), 128, 1, 2, "128x128x36 waves 4x2x1 A=KC/4 B=IM2COL/1 npb=6", None),
    ("128x128 tail split", (25, 64, 28, 28), 256, 1, 1, "128x128x36 waves 4x2x1 A=KC/4 B=IM2COL/1 npb=3", "ksplit=1 tail=52x4"),
    ("128x128 split K", (25, 256, 28, 28), 256, 1, 1, "128x128x36 waves 4x2x1 A=KC/4 B=IM2COL/1 npb=3", "ksplit=2 tail=0x1"),
]


@pytest.mark.parametrize("case", CONV_WINDOW_INSTANCE_CASES, ids=[c[0] for c in CONV_WINDOW_INSTANCE_CASES])
def test_every_conv_window_instance(lib, workspace, case):
    """The pass counts of the LDS-patch kernel that no other test selects (tiny planes: a tile then spans many
    images; dilated and strided patches), and the 128 x 128 tile with a tail split and with a K split, whose
    finishing kernels run one and four workgroups per tile."""
    name, xs, m, d, st, inst, split = case
    announce("conv window instance", name)
    rng = np.random.default_rng([len(name)] + list(xs))
    X = rng.uniform(-1, 1, xs).astype(np.float32)
    Wt = rng.uniform(-1, 1, (m, xs[1], 3, 3)).astype(np.float32)
    Bv = rng.uniform(-1, 1, (m,)).astype(np.float32)
    K = xs[1] * 9
    ref, S = cached(("conv_window_inst", name), lambda: oracle.conv(X, Wt, Bv, (d, d, d, d), (st, st), (d, d), 1, want_scale=True))
    got = host(lib.onnx_conv(dev(X), dev(Wt), dev(Bv), (d, d, d, d), (st, st), (d, d), 1))
    launch = lib.onnx_last_launch()
    assert launch.startswith("conv_window " + inst), (launch, inst)
    assert launch.endswith(split if split and workspace == "workspace" else "ksplit=1 tail=0x1"), launch
    assert rel_err(got, ref) <= REL_TOL
    assert within_rounding_bound(got, ref, S, K + 1)


@pytest.mark.parametrize("case", CONV_INSTANCE_CASES, ids=[c[0] for c in CONV_INSTANCE_CASES])
def test_every_conv_contraction_instance(lib, case):
    """The instances of the contraction kernel only convolutions reach (gather loader, strided 1x1
    loader, image-blocked row-contiguous loader), each tile shape and filter load width once."""
    name, xs, ws_, pads, st, inst = case
    announce("conv instance", name)
    rng = np.random.default_rng([len(name)] + list(xs))
    X = rng.uniform(-1, 1, xs).astype(np.float32)
    Wt = rng.uniform(-1, 1, ws_).astype(np.float32)
    Bv = rng.uniform(-1, 1, (ws_[0],)).astype(np.float32)
    K = ws_[1] * ws_[2] * ws_[3]
    ref, S = cached(("conv_inst", name), lambda: oracle.conv(X, Wt, Bv, pads, st, (1, 1), 1, want_scale=True))
    got = host(lib.onnx_conv(dev(X), dev(Wt), dev(Bv), pads, st, (1, 1), 1))
    assert lib.onnx_last_launch().startswith("contraction " + inst), (lib.onnx_last_launch(), inst)
    assert rel_err(got, ref) <= REL_TOL
    assert within_rounding_bound(got, ref, S, K + 1)
