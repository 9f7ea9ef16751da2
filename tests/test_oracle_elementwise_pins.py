"""Pins for the element-wise / reduction / softmax oracle: hand-worked values, closed forms,
brute force over tiny tensors with plain Python loops, and torch's CPU operators in float64
(independent library routines).  None of the expected values comes from the oracle or the GPU."""
import itertools
import math

import numpy as np
import pytest

from oracle import elementwise as ew


def test_add_paper_example_shape_and_closed_form():
    # the paper's running example adds two 3x4x5 tensors element by element (Section 3)
    a = np.arange(60, dtype=np.float32).reshape(3, 4, 5)
    b = (2 * np.arange(60, dtype=np.float32)).reshape(3, 4, 5)
    y = ew.add(a, b)
    assert y.shape == (3, 4, 5) and y.dtype == np.float64
    for i, j, k in itertools.product(range(3), range(4), range(5)):
        assert y[i, j, k] == 3.0 * (20 * i + 5 * j + k)


@pytest.mark.parametrize("sa,sb", [((2, 3, 4), (3, 1)), ((4,), (2, 1, 4)), ((2, 1, 3), (1, 5, 1)),
                                   ((1,), (3, 2)), ((2, 3), ()), ((5, 1, 1), (1, 6))])
def test_add_broadcasting_brute_force(sa, sb):
    rng = np.random.default_rng(3)
    a = rng.integers(-9, 10, sa).astype(np.float32)
    b = rng.integers(-9, 10, sb).astype(np.float32)
    y = ew.add(a, b)
    rank = max(len(sa), len(sb))
    pa, pb = (1,) * (rank - len(sa)) + tuple(sa), (1,) * (rank - len(sb)) + tuple(sb)
    shape = tuple(max(x, z) for x, z in zip(pa, pb))
    assert y.shape == shape
    ar, br = a.reshape(pa), b.reshape(pb)
    for idx in itertools.product(*[range(n) for n in shape]):
        ia = tuple(0 if pa[d] == 1 else idx[d] for d in range(rank))
        ib = tuple(0 if pb[d] == 1 else idx[d] for d in range(rank))
        assert y[idx] == float(ar[ia]) + float(br[ib])
    with pytest.raises(ValueError):
        ew.add(np.zeros((2, 3), np.float32), np.zeros((4,), np.float32))


def test_unary_hand_values():
    x = np.array([-2.0, -0.5, 0.0, 3.0], np.float32)
    assert ew.relu(x).tolist() == [0.0, 0.0, 0.0, 3.0]
    got = ew.leakyrelu(x, 0.25)
    assert got.tolist() == [-0.5, -0.125, 0.0, 3.0]
    # default slope 0.01 as an fp32 attribute
    assert ew.leakyrelu(np.array([-100.0], np.float32))[0] == -100.0 * float(np.float32(0.01))
    assert ew.absolute(x).tolist() == [2.0, 0.5, 0.0, 3.0]


def test_reducesum_closed_forms_and_shapes():
    n = 1000
    x = np.arange(n, dtype=np.float32)
    assert ew.reducesum(x, None, 0) == n * (n - 1) / 2
    x3 = np.arange(24, dtype=np.float32).reshape(2, 3, 4)
    assert ew.reducesum(x3, [1], 1).shape == (2, 1, 4)
    assert ew.reducesum(x3, [1], 0).shape == (2, 4)
    assert ew.reducesum(x3, [-1, 0], 1).shape == (1, 3, 1)
    assert ew.reducesum(x3, [], 1).shape == (1, 1, 1)
    assert ew.reducesum(x3, [0, 2], 0).tolist() == [sum(12 * i + 4 * j + k for i in range(2) for k in range(4)) for j in range(3)]
    with pytest.raises(ValueError):
        ew.reducesum(x3, [3], 1)
    with pytest.raises(ValueError):
        ew.reducesum(x3, [1, -2], 1)


@pytest.mark.parametrize("axes", [[0], [1], [2], [3], [0, 1], [1, 3], [0, 2, 3], [0, 1, 2, 3], [-1, -3]])
def test_reducesum_brute_force(axes):
    rng = np.random.default_rng(4)
    x = rng.integers(-5, 6, (2, 3, 2, 4)).astype(np.float32)
    ax = sorted(a % 4 for a in axes)
    want = np.zeros([1 if d in ax else x.shape[d] for d in range(4)])
    for idx in itertools.product(*[range(n) for n in x.shape]):
        o = tuple(0 if d in ax else idx[d] for d in range(4))
        want[o] += float(x[idx])
    assert np.array_equal(ew.reducesum(x, axes, 1), want)
    assert np.array_equal(ew.reducesum(x, axes, 0), want.reshape([x.shape[d] for d in range(4) if d not in ax]))
    # ReduceL1 is ReduceSum of Abs (the decomposition of Section 3.4)
    assert np.array_equal(ew.reducel1(x, axes, 1), ew.reducesum(ew.absolute(x).astype(np.float32), axes, 1))


def test_reducel1_hand_value():
    x = np.array([[1.0, -2.0, 3.0], [-4.0, 5.0, -6.0]], np.float32)
    assert ew.reducel1(x, [1], 0).tolist() == [6.0, 15.0]
    assert ew.reducel1(x, [0], 1).tolist() == [[5.0, 7.0, 9.0]]
    assert ew.reducel1(x, None, 0) == 21.0


def test_softmax_closed_forms():
    y = ew.softmax(np.array([0.0, math.log(3.0)], np.float32))
    l3 = float(np.float32(math.log(3.0)))
    assert abs(y[0] - 1.0 / (1.0 + math.exp(l3))) < 1e-15 and abs(y[1] - math.exp(l3) / (1.0 + math.exp(l3))) < 1e-15
    c = ew.softmax(np.full((3, 7), 2.5, np.float32), axis=1)
    assert np.allclose(c, 1.0 / 7.0, rtol=0, atol=1e-16)
    rng = np.random.default_rng(6)
    x = rng.standard_normal((4, 5, 6)).astype(np.float32)
    for axis in (0, 1, 2, -1, -3):
        s = ew.softmax(x, axis)
        assert np.allclose(s.sum(axis=axis), 1.0, rtol=0, atol=1e-14)
        assert np.allclose(ew.softmax(x + np.float32(3.0), axis), s, rtol=1e-6, atol=0)   # shift invariance (fp32 add rounds)
        assert (np.argmax(s, axis=axis) == np.argmax(x, axis=axis)).all()
    # large logits do not overflow
    big = ew.softmax(np.array([1000.0, 1000.0, -1000.0], np.float32))
    assert big.tolist() == [0.5, 0.5, 0.0]
    with pytest.raises(ValueError):
        ew.softmax(x, 3)


def test_against_torch_float64():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(8)
    x = rng.standard_normal((3, 5, 4, 6)).astype(np.float32)
    t = torch.from_numpy(x).double()
    for axis in range(4):
        assert np.allclose(ew.softmax(x, axis), torch.softmax(t, dim=axis).numpy(), rtol=1e-13, atol=0)
    for axes in ([0], [1, 2], [0, 3], [2]):
        assert np.allclose(ew.reducesum(x, axes, 1), t.sum(dim=axes, keepdim=True).numpy(), rtol=1e-13, atol=1e-13)
        assert np.allclose(ew.reducel1(x, axes, 0), t.abs().sum(dim=axes).numpy(), rtol=1e-13, atol=1e-13)
    assert np.array_equal(ew.relu(x), torch.relu(t).numpy())
    assert np.allclose(ew.leakyrelu(x, 0.2), torch.nn.functional.leaky_relu(t, float(np.float32(0.2))).numpy(), rtol=1e-15)
    b = rng.standard_normal((5, 1, 6)).astype(np.float32)
    assert np.array_equal(ew.add(x, b), (t + torch.from_numpy(b).double()).numpy())


def test_round_to_16bit_half_matches_numpy_and_bfloat16_matches_torch():
    """The oracle's one-step rounding to a 16-bit type against two library conversions that round once: numpy's
    double -> float16, and torch's float32 -> bfloat16 on doubles that are float32 values."""
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(21)
    v = np.concatenate([rng.standard_normal(4000) * 10.0 ** rng.integers(-9, 6, 4000),
                        np.ldexp(rng.integers(-3000, 3000, 500).astype(np.float64), -25),       # half's subnormals and their ties
                        np.array([0.0, -0.0, 65504.0, 65519.9, 65520.0, -65520.0, 1e9, np.inf, -np.inf, 2.0 ** -24, 2.0 ** -25, 3 * 2.0 ** -25])])
    with np.errstate(over="ignore"):
        want = v.astype(np.float16).astype(np.float64)
    got = ew.round_to_16bit(v, "f16")
    assert np.array_equal(got, want) and np.array_equal(np.signbit(got), np.signbit(want))
    assert np.isnan(ew.round_to_16bit(np.array([np.nan]), "f16"))[0]
    f = np.concatenate([(rng.standard_normal(4000) * 10.0 ** rng.integers(-30, 30, 4000)).astype(np.float32),
                        np.array([3.3895314e38, 3.4e38, -3.4e38, 1e-40, -1e-40, 9.1e-41, 0.0], dtype=np.float32)])
    want = torch.from_numpy(f).to(torch.bfloat16).double().numpy()
    assert np.array_equal(ew.round_to_16bit(f.astype(np.float64), "bf16"), want)


def test_round_to_16bit_ties_and_error_bound():
    """Hand-worked ties (to the even significand) and, over random doubles, the definition itself in exact rational
    arithmetic: the result is within half a spacing of the input, and on the even neighbour when exactly half away."""
    from fractions import Fraction
    cases = [(1 + 2.0 ** -8, 1.0), (1 + 3 * 2.0 ** -8, 1 + 2.0 ** -6), (1 + 2.0 ** -8 + 2.0 ** -30, 1 + 2.0 ** -7),
             (2.0 ** -134, 0.0), (3 * 2.0 ** -134, 2.0 ** -132), (-(1 + 2.0 ** -8), -1.0), (3.39e38, 3.3895313892515355e38),
             (3.3962e38, np.inf)]
    for v, want in cases:
        assert ew.round_to_16bit(np.array([v]), "bf16")[0] == want, v
    assert ew.round_to_16bit(np.array([1 + 2.0 ** -11]), "f16")[0] == 1.0
    assert ew.round_to_16bit(np.array([1 + 3 * 2.0 ** -11]), "f16")[0] == 1 + 2.0 ** -9
    rng = np.random.default_rng(22)
    for kind, bits, emin in (("f16", 11, -14), ("bf16", 8, -126)):
        v = rng.standard_normal(300) * 10.0 ** rng.integers(-4, 4, 300)
        v[:40] = np.ldexp(rng.integers(1, 1 << 12, 40).astype(np.float64), rng.integers(-20, 5, 40) - 12)   # many exact ties
        r = ew.round_to_16bit(v, kind)
        for x, y in zip(v.tolist(), r.tolist()):
            e = max(math.frexp(x)[1], emin + 1)
            spacing = Fraction(2) ** (e - bits)
            err = abs(Fraction(y) - Fraction(x))
            q = Fraction(y) / spacing
            assert q.denominator == 1 and abs(q) <= 2 ** bits, (kind, x, y)          # a value of the type
            assert err * 2 <= spacing, (kind, x, y)
            if err * 2 == spacing:
                assert q.numerator % 2 == 0, (kind, x, y)


def test_add_16bit_is_the_rounded_exact_sum():
    a = np.array([1.0, 1.0, 256.0, -3.0, 65504.0, 0.0], dtype=np.float64)
    b = np.array([2.0 ** -8, 3 * 2.0 ** -8, 1.0, 3.0, 65504.0, -0.0], dtype=np.float64)
    assert ew.add_16bit(a, b, "bf16").tolist() == [1.0, 1 + 2.0 ** -6, 256.0, 0.0, 131072.0, 0.0]      # 257 ties to 256
    assert ew.add_16bit(a, b, "f16").tolist() == [1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, 257.0, 0.0, np.inf, 0.0]
