"""Pins the CPU oracle to things other than itself (no GPU needed).

The operators are those Section 4.1 of the paper lists as supported (convolution, pooling,
Gemm) plus MatMul from Section 3.4's MulAddToGemmPattern.  Pins used:
  * hand-worked examples stored under tests/golden/;
  * torch's CPU operators in float64 (independent library routines) on random attribute mixes;
  * a second formulation of convolution (explicit zero padding, zero-inserted dilated kernel,
    stride-1 correlation, then subsampling) built from numpy slicing;
  * algebraic identities: 1x1 conv == Gemm, shifted-delta kernels, linearity in the weights,
    grouped conv == concatenation, batch independence, MatMul+Add == Gemm, transposition;
  * the BatchNorm folding identity and the ResNet-50 graph's size (about 100 MB of weights,
    Section 4.2).
"""
import itertools

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
import workloads


def _t64(a):
    return torch.tensor(np.asarray(a), dtype=torch.float64)


# ------------------------------------------------------------------ golden worked examples

def test_golden_conv(golden):
    for c in golden["conv"]:
        X = np.array(c["x"], np.float32).reshape(c["x_shape"])
        W = np.array(c["w"], np.float32).reshape(c["w_shape"])
        B = None if c["b"] is None else np.array(c["b"], np.float32)
        Y = oracle.conv(X, W, B, c["pads"], c["strides"], c["dilations"], c["group"])
        assert list(Y.shape) == c["y_shape"], c["name"]
        assert np.array_equal(Y.ravel(), np.array(c["y"], np.float64)), c["name"]


def test_golden_maxpool(golden):
    for c in golden["maxpool"]:
        X = np.array(c["x"], np.float32).reshape(c["x_shape"])
        Y, I = oracle.maxpool(X, c["kernel"], c["pads"], c["strides"])
        assert list(Y.shape) == c["y_shape"], c["name"]
        assert np.array_equal(Y.ravel(), np.array(c["y"], np.float32)), c["name"]
        assert np.array_equal(I.ravel(), np.array(c["indices"], np.int64)), c["name"]


def test_golden_avgpool(golden):
    for c in golden["avgpool"]:
        X = np.array(c["x"], np.float32).reshape(c["x_shape"])
        Y = oracle.avgpool(X, c["kernel"], c["pads"], c["strides"], 0, c["count_include_pad"])
        assert np.array_equal(Y.ravel(), np.array(c["y"], np.float64)), c["name"]


def test_golden_gemm(golden):
    for c in golden["gemm"]:
        A = np.array(c["a"], np.float32).reshape(c["a_shape"])
        B = np.array(c["b"], np.float32).reshape(c["b_shape"])
        C = np.array(c["c"], np.float32).reshape(c["c_shape"])
        Y = oracle.gemm(A, B, C, c["alpha"], c["beta"], c["transA"], c["transB"], relu=c["relu"])
        assert np.array_equal(Y.ravel(), np.array(c["y"], np.float64)), c["name"]


# ------------------------------------------------------------------ conv vs torch (library routine)

CONV_CASES = [
    # N, C, H, W, M, kH, kW, pads(T,L,B,R), strides, dilations, group
    (2, 4, 7, 6, 6, 3, 2, (1, 0, 2, 1), (2, 1), (1, 2), 2),
    (1, 3, 9, 8, 5, 3, 3, (1, 1, 1, 1), (1, 1), (1, 1), 1),
    (2, 6, 8, 11, 6, 3, 3, (2, 0, 1, 3), (2, 3), (2, 1), 6),
    (1, 8, 5, 5, 4, 1, 1, (0, 0, 0, 0), (2, 2), (1, 1), 4),
    (3, 2, 12, 10, 7, 5, 4, (0, 3, 4, 0), (3, 2), (2, 2), 1),
    (1, 5, 6, 6, 10, 2, 2, (1, 1, 0, 0), (1, 1), (3, 3), 5),
]


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_matches_torch_float64(case):
    N, C, H, W, M, kH, kW, pads, st, dl, g = case
    rng = np.random.default_rng(hash(case) % (2 ** 32))
    X = rng.standard_normal((N, C, H, W)).astype(np.float32)
    Wt = rng.standard_normal((M, C // g, kH, kW)).astype(np.float32)
    B = rng.standard_normal(M).astype(np.float32)
    Y = oracle.conv(X, Wt, B, pads, st, dl, g)
    xp = F.pad(_t64(X), (pads[1], pads[3], pads[0], pads[2]))
    ref = F.conv2d(xp, _t64(Wt), _t64(B), stride=st, dilation=dl, groups=g).numpy()
    assert Y.shape == ref.shape
    np.testing.assert_allclose(Y, ref, rtol=1e-12, atol=1e-12)


def _conv_second_formulation(X, Wt, pads, st, dl, g):
    """Pad explicitly, dilate the kernel by zero insertion, correlate at stride 1 with
    shifted-slice accumulation, then subsample.  Integer data keeps every step exact."""
    N, C, H, W = X.shape
    M, Cg, kH, kW = Wt.shape
    Xp = np.zeros((N, C, H + pads[0] + pads[2], W + pads[1] + pads[3]), np.float64)
    Xp[:, :, pads[0]:pads[0] + H, pads[1]:pads[1] + W] = X
    eH, eW = (kH - 1) * dl[0] + 1, (kW - 1) * dl[1] + 1
    Wd = np.zeros((M, Cg, eH, eW), np.float64)
    Wd[:, :, ::dl[0], ::dl[1]] = Wt
    fH, fW = Xp.shape[2] - eH + 1, Xp.shape[3] - eW + 1
    full = np.zeros((N, M, fH, fW), np.float64)
    Mg = M // g
    for m in range(M):
        grp = m // Mg
        for c in range(Cg):
            for a in range(eH):
                for b in range(eW):
                    if Wd[m, c, a, b] != 0.0:
                        full[:, m] += Wd[m, c, a, b] * Xp[:, grp * Cg + c, a:a + fH, b:b + fW]
    return full[:, :, ::st[0], ::st[1]]


def test_conv_bruteforce_second_formulation_exact():
    rng = np.random.default_rng(11)
    n_checked = 0
    for kH, kW, sH, sW, dH, dW, g in itertools.product((1, 3), (2, 3), (1, 2), (1, 3), (1, 2), (1, 2), (1, 2)):
        N, C, H, W, M = 2, 4, 7, 6, 4
        pads = tuple(int(v) for v in rng.integers(0, 3, size=4))
        X = rng.integers(-4, 5, size=(N, C, H, W)).astype(np.float32)
        Wt = rng.integers(-4, 5, size=(M, C // g, kH, kW)).astype(np.float32)
        if H + pads[0] + pads[2] < (kH - 1) * dH + 1 or W + pads[1] + pads[3] < (kW - 1) * dW + 1:
            continue
        Y = oracle.conv(X, Wt, None, pads, (sH, sW), (dH, dW), g)
        ref = _conv_second_formulation(X, Wt, pads, (sH, sW), (dH, dW), g)
        assert Y.shape == ref.shape
        assert np.array_equal(Y, ref), (kH, kW, sH, sW, dH, dW, g, pads)
        n_checked += 1
    assert n_checked > 100


def test_conv_1x1_equals_gemm():
    rng = np.random.default_rng(5)
    N, C, H, W, M = 3, 7, 5, 4, 6
    X = rng.standard_normal((N, C, H, W)).astype(np.float32)
    Wt = rng.standard_normal((M, C, 1, 1)).astype(np.float32)
    B = rng.standard_normal(M).astype(np.float32)
    Y = oracle.conv(X, Wt, B)
    for n in range(N):
        G = oracle.gemm(Wt.reshape(M, C), X[n].reshape(C, H * W), B.reshape(M, 1))
        np.testing.assert_allclose(Y[n].reshape(M, H * W), G, rtol=0, atol=1e-13)


def test_conv_shifted_delta_kernel_reproduces_input():
    rng = np.random.default_rng(6)
    N, C, H, W = 2, 3, 9, 8
    X = rng.standard_normal((N, C, H, W)).astype(np.float32)
    for (kH, kW, a, b, dH, dW, pads, st) in [
        (3, 3, 1, 1, 1, 1, (1, 1, 1, 1), (1, 1)),       # centred delta: identity
        (3, 3, 0, 2, 2, 1, (1, 0, 3, 2), (1, 1)),
        (2, 4, 1, 3, 1, 2, (0, 2, 1, 4), (2, 3)),
    ]:
        Wt = np.zeros((C, C, kH, kW), np.float32)
        for c in range(C):
            Wt[c, c, a, b] = 1.0
        Y = oracle.conv(X, Wt, None, pads, st, (dH, dW))
        OH, OW = Y.shape[2:]
        ref = np.zeros_like(Y)
        for oh in range(OH):
            for ow in range(OW):
                ih, iw = oh * st[0] - pads[0] + a * dH, ow * st[1] - pads[1] + b * dW
                if 0 <= ih < H and 0 <= iw < W:
                    ref[:, :, oh, ow] = X[:, :, ih, iw]
        assert np.array_equal(Y, ref)
    Wt = np.zeros((C, C, 3, 3), np.float32)
    for c in range(C):
        Wt[c, c, 1, 1] = 1.0
    assert np.array_equal(oracle.conv(X, Wt, None, (1, 1, 1, 1)), X.astype(np.float64))


def test_conv_linear_in_weights_exact_on_integers():
    rng = np.random.default_rng(7)
    X = rng.integers(-4, 5, size=(2, 4, 6, 7)).astype(np.float32)
    W1 = rng.integers(-3, 4, size=(5, 4, 3, 3)).astype(np.float32)
    W2 = rng.integers(-3, 4, size=(5, 4, 3, 3)).astype(np.float32)
    kw = dict(pads=(1, 2, 0, 1), strides=(2, 1), dilations=(1, 2))
    lhs = oracle.conv(X, 2 * W1 - 3 * W2, None, **kw)
    rhs = 2 * oracle.conv(X, W1, None, **kw) - 3 * oracle.conv(X, W2, None, **kw)
    assert np.array_equal(lhs, rhs)


def test_conv_group_is_concatenation_and_batch_independent():
    rng = np.random.default_rng(8)
    N, C, M, g = 3, 6, 9, 3
    X = rng.standard_normal((N, C, 6, 5)).astype(np.float32)
    Wt = rng.standard_normal((M, C // g, 3, 3)).astype(np.float32)
    B = rng.standard_normal(M).astype(np.float32)
    kw = dict(pads=(1, 1, 1, 1), strides=(1, 2))
    Y = oracle.conv(X, Wt, B, group=g, **kw)
    Cg, Mg = C // g, M // g
    for i in range(g):
        part = oracle.conv(X[:, i * Cg:(i + 1) * Cg], Wt[i * Mg:(i + 1) * Mg], B[i * Mg:(i + 1) * Mg], **kw)
        assert np.array_equal(Y[:, i * Mg:(i + 1) * Mg], part)
    for n in range(N):
        assert np.array_equal(Y[n:n + 1], oracle.conv(X[n:n + 1], Wt, B, group=g, **kw))


def test_conv_epilogue_residual_relu_and_scale():
    rng = np.random.default_rng(9)
    X = rng.standard_normal((2, 3, 6, 6)).astype(np.float32)
    Wt = rng.standard_normal((4, 3, 3, 3)).astype(np.float32)
    B = rng.standard_normal(4).astype(np.float32)
    R = rng.standard_normal((2, 4, 6, 6)).astype(np.float32)
    base = oracle.conv(X, Wt, B, (1, 1, 1, 1))
    Y, S = oracle.conv(X, Wt, B, (1, 1, 1, 1), residual=R, relu=True, want_scale=True)
    np.testing.assert_allclose(Y, np.maximum(base + R.astype(np.float64), 0.0), rtol=0, atol=1e-13)
    assert (Y >= 0).all() and (Y == 0).any() and (Y > 0).any()
    Sref = oracle.conv(np.abs(X), np.abs(Wt), np.abs(B), (1, 1, 1, 1), residual=np.abs(R))
    np.testing.assert_allclose(S, Sref, rtol=1e-13)
    assert (S >= np.abs(base + R) - 1e-12).all()


def test_conv_rejects_bad_arguments():
    X = np.zeros((1, 4, 5, 5), np.float32)
    with pytest.raises(ValueError):
        oracle.conv(X, np.zeros((6, 2, 3, 3), np.float32), group=3)        # group does not divide C
    with pytest.raises(ValueError):
        oracle.conv(X, np.zeros((6, 4, 3, 3), np.float32), strides=(0, 1))
    with pytest.raises(ValueError):
        oracle.conv(X, np.zeros((6, 4, 7, 7), np.float32))                 # window larger than input
    with pytest.raises(ValueError):
        oracle.conv(X, np.zeros((6, 4, 3, 3), np.float32), pads=(-1, 0, 0, 0))


# ------------------------------------------------------------------ gemm / matmul

@pytest.mark.parametrize("transA,transB", [(0, 0), (0, 1), (1, 0), (1, 1)])
@pytest.mark.parametrize("cshape", [None, (), (5,), (1, 5), (4, 1), (4, 5), (1, 1)])
def test_gemm_matches_numpy_float64(transA, transB, cshape):
    rng = np.random.default_rng(21)
    M, N, K = 4, 5, 7
    A = rng.standard_normal((K, M) if transA else (M, K)).astype(np.float32)
    B = rng.standard_normal((N, K) if transB else (K, N)).astype(np.float32)
    C = None if cshape is None else rng.standard_normal(cshape).astype(np.float32)
    alpha, beta = 0.75, -1.5
    Y = oracle.gemm(A, B, C, alpha, beta, transA, transB)
    a = A.astype(np.float64).T if transA else A.astype(np.float64)
    b = B.astype(np.float64).T if transB else B.astype(np.float64)
    ref = alpha * (a @ b)
    if C is not None:
        ref = ref + beta * np.broadcast_to(C.astype(np.float64), (M, N))
    np.testing.assert_allclose(Y, ref, rtol=1e-13, atol=1e-13)


def test_gemm_transpose_identities_and_matmul_add_rewrite():
    """Section 3.4: Add(MatMul(m1, m2), m3) may be replaced by Gemm(m1, m2, m3)."""
    rng = np.random.default_rng(22)
    A = rng.integers(-4, 5, size=(6, 9)).astype(np.float32)
    B = rng.integers(-4, 5, size=(9, 5)).astype(np.float32)
    C = rng.integers(-4, 5, size=(6, 5)).astype(np.float32)
    fused = oracle.gemm(A, B, C)
    assert np.array_equal(fused, oracle.matmul(A, B) + C.astype(np.float64))
    assert np.array_equal(fused, oracle.gemm(A, np.ascontiguousarray(B.T), C, transB=1))
    assert np.array_equal(fused, oracle.gemm(np.ascontiguousarray(A.T), B, C, transA=1))
    assert np.array_equal(fused, oracle.gemm(np.ascontiguousarray(A.T), np.ascontiguousarray(B.T), C, transA=1, transB=1))
    Y, S = oracle.gemm(A, B, C, alpha=-2.0, beta=0.5, relu=True, want_scale=True)
    assert np.array_equal(Y, np.maximum(-2.0 * oracle.matmul(A, B) + 0.5 * C, 0))
    assert np.array_equal(S, 2.0 * oracle.matmul(np.abs(A), np.abs(B)) + 0.5 * np.abs(C))


def test_gemm_rejects_bad_shapes():
    A = np.zeros((3, 4), np.float32)
    with pytest.raises(ValueError):
        oracle.gemm(A, np.zeros((5, 6), np.float32))
    with pytest.raises(ValueError):
        oracle.gemm(A, np.zeros((4, 6), np.float32), np.zeros((2, 6), np.float32))
    with pytest.raises(ValueError):
        oracle.gemm(A, np.zeros((4, 6), np.float32), np.zeros((3, 5), np.float32))


@pytest.mark.parametrize("sa,sb", [
    ((5, 4), (4, 6)), ((3, 2, 5, 4), (2, 4, 6)), ((2, 5, 4), (3, 1, 4, 6)), ((4,), (4, 6)),
    ((5, 4), (4,)), ((4,), (4,)), ((3, 1, 5, 4), (1, 2, 4, 6)), ((2, 3, 5, 4), (4, 6)),
    ((4,), (2, 3, 4, 6)), ((2, 3, 5, 4), (4,)),
])
def test_matmul_matches_numpy_broadcast(sa, sb):
    rng = np.random.default_rng(23)
    A = rng.standard_normal(sa).astype(np.float32)
    B = rng.standard_normal(sb).astype(np.float32)
    Y = oracle.matmul(A, B)
    ref = np.matmul(A.astype(np.float64), B.astype(np.float64))
    assert Y.shape == ref.shape
    np.testing.assert_allclose(Y, ref, rtol=1e-13, atol=1e-13)


def test_matmul_is_a_loop_of_2d_products_and_rejects_mismatch():
    rng = np.random.default_rng(24)
    A = rng.integers(-4, 5, size=(2, 3, 4, 5)).astype(np.float32)
    B = rng.integers(-4, 5, size=(3, 5, 6)).astype(np.float32)
    Y = oracle.matmul(A, B)
    for i in range(2):
        for j in range(3):
            assert np.array_equal(Y[i, j], oracle.gemm(A[i, j], B[j]))
    with pytest.raises(ValueError):
        oracle.matmul(np.zeros((2, 3, 4), np.float32), np.zeros((3, 4, 5), np.float32))
    with pytest.raises(ValueError):
        oracle.matmul(np.zeros((3, 4), np.float32), np.zeros((5, 6), np.float32))


# ------------------------------------------------------------------ pools

POOL_CASES = [
    # N, C, H, W, k, pads, strides, dil, ceil
    (2, 3, 9, 8, (3, 3), (1, 1, 1, 1), (2, 2), (1, 1), 0),
    (1, 2, 10, 7, (2, 3), (0, 1, 0, 1), (2, 1), (1, 1), 0),
    (2, 2, 11, 11, (3, 3), (1, 1, 1, 1), (2, 2), (1, 1), 1),
    (1, 3, 12, 9, (3, 2), (0, 0, 0, 0), (3, 2), (2, 2), 0),
    (1, 1, 7, 7, (2, 2), (0, 0, 0, 0), (2, 2), (1, 1), 1),
    (1, 2, 13, 10, (3, 3), (1, 1, 1, 1), (1, 1), (2, 3), 0),
]


@pytest.mark.parametrize("case", POOL_CASES)
def test_maxpool_matches_torch(case):
    N, C, H, W, k, pads, st, dl, ceil = case
    assert pads[0] == pads[2] and pads[1] == pads[3]          # torch takes symmetric pads only
    rng = np.random.default_rng(31)
    # few distinct values so that ties are common
    X = rng.integers(-3, 4, size=(N, C, H, W)).astype(np.float32)
    Y, I = oracle.maxpool(X, k, pads, st, dl, ceil)
    yt, it = F.max_pool2d(torch.tensor(X), k, st, (pads[0], pads[1]), dl, ceil_mode=bool(ceil),
                          return_indices=True)
    assert Y.shape == tuple(yt.shape)
    assert np.array_equal(Y, yt.numpy())
    assert np.array_equal(X.ravel()[I], Y)                     # the index addresses the maximum
    plane = (np.arange(N * C) * H * W).reshape(N, C, 1, 1)
    # torch numbers positions within one H x W plane; it breaks ties as the oracle does
    assert np.array_equal(I - plane, it.numpy())


def test_maxpool_asymmetric_pads_bruteforce():
    rng = np.random.default_rng(32)
    X = rng.integers(-3, 4, size=(2, 2, 6, 7)).astype(np.float32)
    k, pads, st = (3, 2), (2, 0, 1, 1), (2, 2)
    Y, I = oracle.maxpool(X, k, pads, st)
    N, C, H, W = X.shape
    Xp = np.full((N, C, H + 3, W + 1), -np.inf, np.float32)
    Xp[:, :, 2:2 + H, 0:W] = X
    OH, OW = (H + 3 - 3) // 2 + 1, (W + 1 - 2) // 2 + 1
    assert Y.shape == (N, C, OH, OW)
    for oh in range(OH):
        for ow in range(OW):
            win = Xp[:, :, oh * 2:oh * 2 + 3, ow * 2:ow * 2 + 2].reshape(N, C, -1)
            assert np.array_equal(Y[:, :, oh, ow], win.max(-1))
            first = win.argmax(-1)                             # numpy returns the first maximum
            ih, iw = oh * 2 - 2 + first // 2, ow * 2 + first % 2
            flat = (np.arange(N)[:, None] * C + np.arange(C)[None, :]) * H * W + ih * W + iw
            assert np.array_equal(I[:, :, oh, ow], flat)


def test_maxpool_identity_window():
    rng = np.random.default_rng(33)
    X = rng.standard_normal((2, 3, 4, 5)).astype(np.float32)
    Y, I = oracle.maxpool(X, (1, 1))
    assert np.array_equal(Y, X) and np.array_equal(I.ravel(), np.arange(X.size))
    with pytest.raises(ValueError):
        oracle.maxpool(X, (2, 2), pads=(2, 0, 0, 0))            # a window made of padding only


@pytest.mark.parametrize("case", POOL_CASES)
@pytest.mark.parametrize("cip", [0, 1])
def test_avgpool_matches_torch(case, cip):
    N, C, H, W, k, pads, st, dl, ceil = case
    if dl != (1, 1):
        pytest.skip("AveragePool has no dilation here")
    rng = np.random.default_rng(34)
    X = rng.standard_normal((N, C, H, W)).astype(np.float32)
    Y = oracle.avgpool(X, k, pads, st, ceil, cip)
    ref = F.avg_pool2d(_t64(X), k, st, (pads[0], pads[1]), ceil_mode=bool(ceil),
                       count_include_pad=bool(cip)).numpy()
    assert Y.shape == ref.shape
    np.testing.assert_allclose(Y, ref, rtol=1e-13, atol=1e-13)


def test_avgpool_global_and_constant():
    rng = np.random.default_rng(35)
    X = rng.standard_normal((2, 5, 7, 7)).astype(np.float32)
    G = oracle.avgpool(X, None)
    assert G.shape == (2, 5, 1, 1)
    np.testing.assert_allclose(G[:, :, 0, 0], X.astype(np.float64).mean(axis=(2, 3)), rtol=1e-13)
    Cst = np.full((1, 2, 6, 6), 3.25, np.float32)
    Y = oracle.avgpool(Cst, (3, 3), (1, 1, 1, 1), (2, 2), 0, 0)
    assert np.array_equal(Y, np.full(Y.shape, 3.25))


def test_window_out_formula():
    assert oracle.window_out(224, 7, 3, 3, 2) == 112
    assert oracle.window_out(112, 3, 1, 1, 2) == 56
    assert oracle.window_out(28, 3, 2, 2, 1, 2) == 28
    assert oracle.window_out(14, 3, 0, 0, 3) == 4
    assert oracle.window_out(7, 2, 0, 0, 2, 1, 1) == 4
    assert oracle.window_out(7, 2, 0, 0, 2, 1, 0) == 3
    assert oracle.window_out(4, 2, 1, 1, 2, 1, 1) == 3          # ceil would give 3 and the last window starts inside
    assert oracle.window_out(3, 2, 1, 1, 2, 1, 1) == 2          # would start in the trailing padding: dropped
    assert oracle.window_out(2, 5, 1, 1, 1) == -1


# ------------------------------------------------------------------ workloads

def test_batchnorm_folding_identity():
    """conv followed by an explicit BatchNorm (double) equals the conv with folded weights."""
    r = np.random.default_rng(41)
    wf, bf, raw = workloads._folded_conv(r, 6, 4, 3)
    X = r.standard_normal((2, 4, 8, 8)).astype(np.float32)
    y = oracle.conv(X, raw["w"], None, (1, 1, 1, 1))
    s = raw["gamma"] / np.sqrt(raw["var"] + workloads.BN_EPS)
    bn = (y - raw["mean"][None, :, None, None]) * s[None, :, None, None] + raw["beta"][None, :, None, None]
    folded = oracle.conv(X, wf, bf, (1, 1, 1, 1))
    np.testing.assert_allclose(folded, bn, rtol=0, atol=5e-6 * np.abs(bn).max())


def test_resnet50_graph_size_matches_paper():
    """Section 4.2: the ResNet50 model is about 100 MB including weights."""
    m = workloads.resnet50(1)
    st = workloads.graph_stats(m)
    assert sum(1 for n in m["graph"] if n["op"] == "conv") == 53
    assert st["params"] == 25530472
    assert 95e6 < st["params"] * 4 < 105e6
    assert st["macs"] == 4089184256
    assert st["shapes"]["logits"] == (1, 1000)


def test_small_cnn_chain_shapes_and_values():
    from oracle import chain
    m = workloads.small_cnn()
    env, exact = chain.run(m)
    assert env["c1"].shape == (1, 8, 28, 28) and env["p1"].shape == (1, 8, 14, 14)
    assert env["c2"].shape == (1, 16, 14, 14) and env["p2"].shape == (1, 16, 4, 4)
    assert exact["logits"].shape == (1, 10)
    # the same chain through torch's CPU operators in double
    x = _t64(m["inputs"]["x"])
    w = {k: _t64(v) for k, v in m["weights"].items()}
    t = F.relu(F.conv2d(x, w["w1"], w["b1"], padding=2)).float().double()
    t = F.max_pool2d(t, 2, 2)
    t = F.relu(F.conv2d(t, w["w2"], w["b2"], padding=2)).float().double()
    t = F.max_pool2d(t, 3, 3).reshape(1, 256)
    ref = (t @ w["wg"] + w["bg"]).numpy()
    np.testing.assert_allclose(exact["logits"], ref, rtol=1e-12, atol=1e-12)


def test_bf16_input_encoding_matches_torch_and_the_format_definition():
    """The generator's fp32 -> bfloat16 encoding (input preparation for the 16-bit Gemm cases, also
    used to state the expected rounding of 16-bit results) against an independent library routine
    (torch's conversion) and against the format's definition: the upper 16 bits of the binary32
    pattern, round to nearest, ties to even."""
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(16)
    x = np.concatenate([rng.standard_normal(20000) * 10.0 ** rng.integers(-20, 20, 20000),
                        [0.0, -0.0, 1.0, -1.0, 65504.0, 3.0e38, 1e-40, np.inf, -np.inf]]).astype(np.float32)
    bits = workloads.to_bf16_bits(x)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, want)
    assert np.array_equal(workloads.from_bf16_bits(bits), torch.from_numpy(x).to(torch.bfloat16).float().numpy())
    # ties: a pattern exactly half way between two bfloat16 values goes to the one with an even last bit
    half = np.array([0x3F808000, 0x3F818000, 0x3F800001 | 0x8000, 0x3F807FFF], dtype=np.uint32).view(np.float32)
    assert list(workloads.to_bf16_bits(half)) == [0x3F80, 0x3F82, 0x3F81, 0x3F80]
    # decoding is exact: every bfloat16 pattern round-trips
    allb = np.arange(0x0000, 0x7F80, dtype=np.uint16)
    assert np.array_equal(workloads.to_bf16_bits(workloads.from_bf16_bits(allb)), allb)
