"""Comparison helpers shared by the CPU and GPU tests (no operator arithmetic)."""
import numpy as np

REL_TOL = 1e-4          # the stated fp32 gate: max relative error against the fp64 oracle
EPS32 = 2.0 ** -24      # unit roundoff of fp32


def rel_err(got, ref):
    """max_i |g_i - r_i| / max(|r_i|, rms(r)).

    A plain element-wise relative error is unbounded where the exact result is
    (nearly) zero because of cancellation, whatever the summation order; so each
    element's error is measured against its own magnitude or the tensor's RMS,
    whichever is larger."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(ref * ref)))
    den = np.maximum(np.abs(ref), rms)
    den = np.where(den == 0.0, 1.0, den)
    return float(np.max(np.abs(got - ref) / den))


def within_rounding_bound(got, ref, scale, terms):
    """Component-wise a-priori bound every correct fp32 evaluation satisfies, whatever its
    summation order: |g - r| <= (terms + 3) * 2^-24 * S with S = sum |a||b| + |bias| + ..."""
    got = np.asarray(got, dtype=np.float64)
    bound = (terms + 3) * EPS32 * np.asarray(scale, dtype=np.float64) * 1.01 + 1e-30
    return bool(np.all(np.abs(got - np.asarray(ref, dtype=np.float64)) <= bound))
