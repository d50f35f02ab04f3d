"""Pins for the oracle's flatten plan (arXiv 2402.17985 Sec. 4.1 Eq. 2-3, Sec. 5.1 padding)."""
import json
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import fq_oracle as O


def _cases(golden_dir):
    with open(os.path.join(golden_dir, "plan_cases.json")) as f:
        return json.load(f)["cases"]


def test_hand_derived_plans(golden_dir):
    for c in _cases(golden_dir):
        src, rep, kp, kpad = O.plan(np.array(c["chmax"], np.float32), c["T"], c["align"])
        assert kp == c["Kprime"], c["name"]
        assert kpad == c["Kpad"], c["name"]
        assert src[:kp].tolist() == c["src_head"], c["name"]
        assert rep[:kp].tolist() == c["rep_head"], c["name"]
        assert (src[kp:] == -1).all() and (rep[kp:] == 0).all(), c["name"]
        assert len(src) == kpad and len(rep) == kpad


@pytest.mark.parametrize("seed", range(6))
def test_closed_form_channel_count_exact_rational(seed):
    """K' = K + sum_j (ceil(max_j / T) - 1), evaluated in exact rational arithmetic (Eq. 2)."""
    rng = np.random.default_rng(seed)
    K = int(rng.integers(1, 300))
    chmax = np.abs(rng.standard_normal(K)).astype(np.float32)
    chmax[rng.integers(0, K, max(1, K // 20))] *= np.float32(rng.uniform(5, 90))
    T = np.float32(rng.uniform(0.3, 3.0))
    align = int(rng.choice([1, 2, 32, 64]))
    src, rep, kp, kpad = O.plan(chmax, float(T), align)
    n = []
    for c in chmax:
        r = Fraction(float(c)) / Fraction(float(T))
        n.append(max(1, -((-r.numerator) // r.denominator)))
    n = np.array(n)
    assert kp == K + int((n - 1).sum())
    assert kpad % align == 0 and 0 <= kpad - kp < align
    # layout (Eq. 3): identity head, appended extras grouped by channel in increasing order
    assert (src[:K] == np.arange(K)).all()
    tail = src[K:kp]
    assert (np.diff(tail) >= 0).all()
    assert (np.bincount(src[:kp], minlength=K) == n).all()
    assert (rep[:kp] == n[src[:kp]]).all()
    assert (src[kp:] == -1).all() and (rep[kp:] == 0).all()
    # Eq. 3 offset of channel j's block: C + sum_{k<j} E_k
    off = K + np.concatenate([[0], np.cumsum(n - 1)[:-1]])
    for j in np.nonzero(n > 1)[0]:
        assert (src[off[j]:off[j] + n[j] - 1] == j).all()


def test_exact_multiple_gets_no_empty_channel():
    # max_j = k*T exactly -> k copies each holding exactly T (reading of Eq. 2 at multiples)
    for k in (1, 2, 3, 17):
        src, rep, kp, _ = O.plan(np.array([k * 0.75], np.float32), 0.75, 1)
        assert kp == k and (rep[:kp] == k).all()
    # one ulp above a multiple needs one more copy
    c = np.nextafter(np.float32(3 * 0.75), np.float32(10))
    _, rep, kp, _ = O.plan(np.array([c], np.float32), 0.75, 1)
    assert kp == 4


def test_bad_arguments_are_rejected():
    good = np.array([1.0, 2.0], np.float32)
    for T in (0.0, -1.0, float("nan"), float("inf")):
        with pytest.raises(O.OracleError):
            O.plan(good, T, 32)
    for bad in ([1.0, float("nan")], [1.0, -0.5], [float("inf"), 1.0]):
        with pytest.raises(O.OracleError):
            O.plan(np.array(bad, np.float32), 1.0, 32)
