"""CPU oracle for the element-wise, reduction and softmax operators (test infrastructure only).

Plain numpy in double precision, each function the operator's definition written out:
nothing here is used by the GPU library, and nothing here uses it.  The operators are the ones
the paper walks through next to the contractions: element-wise Add (the running example of
Section 3), Relu / LeakyRelu (the operator definition shown in Section 3.1), Abs and ReduceSum
(the two halves of the ReduceL1 decomposition of Section 3.4), and Softmax on the classifier's
logits.
"""
import numpy as np


def _f64(a):
    return np.asarray(a, dtype=np.float32).astype(np.float64)


def add(a, b):
    """ONNX Add: C = A + B with multidirectional (numpy-style) broadcasting: shapes are aligned
    at their last axis, each pair of extents is equal or one of them is 1."""
    return _f64(a) + _f64(b)


def round_to_16bit(v, kind):
    """The values of the 16-bit type ("f16": IEEE half, 11 significant bits, exponents -14..15;
    "bf16": bfloat16, 8 significant bits, exponents -126..127) nearest to the doubles `v`, ties to
    the even significand, overflow to infinity: one rounding, straight from the double.  Returned
    as doubles (each exactly representable in the type)."""
    v = np.asarray(v, dtype=np.float64)
    bits, emin, emax = (11, -14, 15) if kind == "f16" else (8, -126, 127)
    with np.errstate(all="ignore"):
        m, e = np.frexp(v)                                   # v = m 2^e, 0.5 <= |m| < 1
        e = np.maximum(e, emin + 1)                          # below the normal range the spacing stays 2^(emin - bits + 1)
        q = np.rint(np.ldexp(v, bits - e))                   # rint rounds halves to even; |q| <= 2^bits
        r = np.ldexp(q, e - bits)
        big = np.ldexp(2.0 - 2.0 ** (1 - bits), emax)        # largest finite value of the type
        r = np.where(np.abs(r) > big, np.sign(v) * np.inf, r)
    return np.where(np.isfinite(v), r, v)


def add_16bit(a, b, kind):
    """ONNX Add on tensors of a 16-bit type: the exact sum (two 16-bit addends: exact in double)
    rounded once to the type."""
    return round_to_16bit(np.asarray(a, dtype=np.float64) + np.asarray(b, dtype=np.float64), kind)


def relu(x):
    """ONNX Relu: y = max(0, x)."""
    x = _f64(x)
    return np.where(x > 0.0, x, 0.0)


def leakyrelu(x, alpha=0.01):
    """ONNX LeakyRelu: y = x for x >= 0, alpha * x otherwise (alpha is an fp32 attribute,
    default 0.01)."""
    x = _f64(x)
    return np.where(x >= 0.0, x, float(np.float32(alpha)) * x)


def absolute(x):
    """ONNX Abs: y = |x|."""
    return np.abs(_f64(x))


def _axes(rank, axes):
    if axes is None or len(axes) == 0:
        return tuple(range(rank))
    out = []
    for a in axes:
        a = int(a)
        if not -rank <= a < rank:
            raise ValueError("axis %d out of range for rank %d" % (a, rank))
        out.append(a % rank)
    if len(set(out)) != len(out):
        raise ValueError("duplicate axis")
    return tuple(sorted(out))


def reducesum(x, axes=None, keepdims=1):
    """ONNX ReduceSum: sum over the listed axes (all axes when none are given); the reduced
    axes stay as extents of 1 when keepdims is set, else they are removed."""
    x = _f64(x)
    return np.sum(x, axis=_axes(x.ndim, axes), keepdims=bool(keepdims))


def reducel1(x, axes=None, keepdims=1):
    """ONNX ReduceL1: sum of absolute values over the listed axes."""
    x = _f64(x)
    return np.sum(np.abs(x), axis=_axes(x.ndim, axes), keepdims=bool(keepdims))


def softmax(x, axis=-1):
    """ONNX Softmax along one axis: y_i = exp(x_i - m) / sum_j exp(x_j - m), m = max_j x_j
    (the shift does not change the value; it is how the definition is evaluated without
    overflow)."""
    x = _f64(x)
    if not -x.ndim <= axis < x.ndim:
        raise ValueError("axis out of range")
    m = np.max(x, axis=axis, keepdims=True)
    e = np.exp(x - m)
    return e / np.sum(e, axis=axis, keepdims=True)
