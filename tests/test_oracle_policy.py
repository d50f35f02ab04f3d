"""Pins for the oracle's offline policy helpers (arXiv 2402.17985 Sec. 4.2: Eq. 5 smoothing,
Eq. 6-7 truncation threshold)."""
import math

import numpy as np
import pytest

from oracle import fq_oracle as O


def test_threshold_hand_cases():
    # Eq. 6-7 by hand.  [1,2,3,4,100]: Q1 = 2, Q3 = 4, IQR = 2 -> fences [-1, 7]; clipped maxima
    # [1,2,3,4,7], mean 3.4; beta = 1.3 -> T = 4.42.  The outlier moved T from 28.6 to 4.42.
    assert O.threshold_boxplot([1, 2, 3, 4, 100], 1.3) == np.float32(4.42)
    # [1,2,3,4]: Q1 = 1.75, Q3 = 3.25 (linear interpolation), fences [-0.5, 5.5]: nothing clipped,
    # mean 2.5 -> T = 3.25
    assert O.threshold_boxplot([4, 1, 3, 2], 1.3) == np.float32(3.25)
    # a single channel, and equal channels: no spread, T = beta * value
    assert O.threshold_boxplot([2.0], 1.5) == np.float32(3.0)
    assert O.threshold_boxplot([2.0] * 7, 1.0) == np.float32(2.0)
    # low outliers are pulled up to the lower fence: [0,10,10,10,10,10,10,10,10]: Q1 = Q3 = 10 -> all clipped to 10
    assert O.threshold_boxplot([0] + [10] * 8, 1.0) == np.float32(10.0)


@pytest.mark.parametrize("seed", range(4))
def test_threshold_against_numpy_quartiles(seed):
    rng = np.random.default_rng(seed)
    K = int(rng.integers(5, 400))
    c = np.abs(rng.standard_normal(K)).astype(np.float32) * 3
    c[rng.integers(0, K, 3)] *= 50
    q1, q3 = np.percentile(c.astype(np.float64), [25, 75])          # library quartiles
    lo, hi = q1 - 1.5 * (q3 - q1), q3 + 1.5 * (q3 - q1)
    want = np.float32(1.3 * np.clip(c.astype(np.float64), lo, hi).mean())
    got = O.threshold_boxplot(c, 1.3)
    assert abs(float(got) - float(want)) <= 2e-7 * float(want)
    # clipping can only lower the mean when the outliers are high
    assert float(got) <= 1.3 * float(c.astype(np.float64).mean()) * (1 + 1e-6)


def test_smoothing_hand_values_and_symmetry():
    # K = 2, maxima [1, 3]: mu = 2, sigma = 1 -> z = -1, +1.  Weight maxima equal to mu -> Sigmoid(0) = 1/2.
    # alpha = 1: s = Sigmoid(z) = 1/(1+e), e/(1+e); they sum to 1.
    s = O.smooth_scales([1, 3], [2, 2], 1.0)
    assert abs(float(s[0]) - 1.0 / (1.0 + math.e)) < 1e-7 and abs(float(s[1]) - math.e / (1.0 + math.e)) < 1e-7
    assert abs(float(s[0]) + float(s[1]) - 1.0) < 1e-7
    # alpha = 0: only the weight term: 1 / Sigmoid(0) = 2
    assert O.smooth_scales([1, 3], [2, 2], 0.0).tolist() == [2.0, 2.0]
    # alpha = 1/2: sqrt(Sigmoid(z_x)) / sqrt(1/2)
    s = O.smooth_scales([1, 3], [2, 2], 0.5)
    assert abs(float(s[1]) - math.sqrt(2 * math.e / (1 + math.e))) < 1e-6
    # no spread: s = 1
    assert O.smooth_scales([5, 5, 5], [1, 2, 3], 0.5).tolist() == [1.0, 1.0, 1.0]


def test_smoothing_keeps_the_product_and_flattens_outliers():
    """Smooth(X, W) = (X diag(s)^-1, diag(s) W) leaves X W unchanged and shrinks the large channels."""
    rng = np.random.default_rng(3)
    M, K, N = 20, 64, 9
    X = rng.standard_normal((M, K)).astype(np.float32)
    X[:, [5, 40]] *= 60
    W = (rng.standard_normal((N, K)) / 8).astype(np.float32)
    cx, cw = np.abs(X).max(axis=0), np.abs(W).max(axis=0)
    s = O.smooth_scales(cx, cw, 0.5).astype(np.float64)
    Xs, Ws = X / s[None, :], W * s[None, :]
    np.testing.assert_allclose(Xs @ Ws.T, X.astype(np.float64) @ W.astype(np.float64).T, rtol=1e-9, atol=1e-9)
    assert (s > 0).all()
    # the outlier channels get the largest divisors
    assert set(np.argsort(s)[-2:].tolist()) == {5, 40}
    assert np.abs(Xs).max() < np.abs(X).max()


def test_policy_bad_arguments():
    with pytest.raises(O.OracleError):
        O.threshold_boxplot([1, -1], 1.3)
    with pytest.raises(O.OracleError):
        O.threshold_boxplot([1, 2], 0.0)
    with pytest.raises(O.OracleError):
        O.smooth_scales([1, 2], [1, 2], 1.5)


def test_channel_absmax_hand_case_and_library():
    """Calibration statistic: hand case, then NumPy's reduction on random data, then the running form."""
    X = np.array([[1.0, -7.0, 0.0], [-3.0, 2.0, 0.0]], dtype=np.float32)
    assert O.channel_absmax(X).tolist() == [3.0, 7.0, 0.0]
    assert O.channel_absmax(X, prev=np.array([5.0, 1.0, 0.5], np.float32)).tolist() == [5.0, 7.0, 0.5]
    rng = np.random.default_rng(3)
    A = rng.standard_normal((37, 53)).astype(np.float32)
    B = (rng.standard_normal((11, 53)) * 3).astype(np.float32)
    np.testing.assert_array_equal(O.channel_absmax(A), np.abs(A).max(axis=0))
    np.testing.assert_array_equal(O.channel_absmax(B, prev=O.channel_absmax(A)),
                                  np.abs(np.concatenate([A, B])).max(axis=0))
