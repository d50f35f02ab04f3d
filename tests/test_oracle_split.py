"""Pins for the oracle's second split rule and two-sided flattening (arXiv 2402.17985, Sec. 4.1):
Eq. 3 as printed ("peel": floor(|x|/T) slots of T, then the remainder) and flattening of the weights'
own large channels (last paragraph of Sec. 4.1).  Hand-derived values, the X'W' = XW identity in
float64 against NumPy, bounds that follow from the construction, and reductions to functions that
are pinned elsewhere."""
import numpy as np
import pytest

from oracle import fq_oracle as O


def test_plan_xw_hand_case():
    # nx = ceil([1,5,1]/2) = [1,3,1]; nw = ceil([.3,.5,.1]/.25) = [2,2,1]; slots per channel 2, 6, 1
    src, rx, rw, od, kp, kpad = O.plan_xw([1, 5, 1], 2.0, [0.3, 0.5, 0.1], 0.25, align=4)
    assert (kp, kpad) == (9, 12)
    assert src.tolist() == [0, 1, 2, 0, 1, 1, 1, 1, 1, -1, -1, -1]
    assert rx.tolist() == [1, 3, 1, 1, 3, 3, 3, 3, 3, 0, 0, 0]
    assert rw.tolist() == [2, 2, 1, 2, 2, 2, 2, 2, 2, 0, 0, 0]
    assert od.tolist() == [0, 0, 0, 1, 1, 2, 3, 4, 5, 0, 0, 0]


@pytest.mark.parametrize("seed", range(5))
def test_plan_xw_without_weights_is_the_one_sided_plan(seed):
    rng = np.random.default_rng(seed)
    K = int(rng.integers(1, 300))
    ch = (np.abs(rng.standard_normal(K)) * rng.choice([1, 1, 1, 30], K)).astype(np.float32)
    T = float(np.float32(rng.uniform(0.5, 3)))
    src, rx, rw, od, kp, kpad = O.plan_xw(ch, T, align=32)
    s1, r1, kp1, kpad1 = O.plan(ch, T, align=32)
    assert (kp, kpad) == (kp1, kpad1)
    np.testing.assert_array_equal(src, s1)
    np.testing.assert_array_equal(rx, r1)
    assert (rw[:kp] == 1).all() and (rw[kp:] == 0).all()
    # ordinals: 0 at the original position, then 1, 2, ... through the channel's appended block
    for j in range(K):
        slots = np.flatnonzero(src == j)
        assert slots[0] == j and od[slots].tolist() == list(range(len(slots)))


@pytest.mark.parametrize("seed", range(4))
def test_two_sided_flatten_keeps_the_product_and_bounds(seed):
    """x*w = sum over nx*nw slots of (x/nx)(w/nw): X'W'^T = XW^T in float64, max|x'| <= T_x, max|w'| <= T_w."""
    rng = np.random.default_rng(100 + seed)
    M, K, N = 9, 40, 7
    X = (rng.standard_normal((M, K)) * rng.choice([1, 1, 20], K)).astype(np.float32)
    W = (rng.standard_normal((N, K)) * 0.05 * rng.choice([1, 1, 6], K)).astype(np.float32)
    cx, cw = np.abs(X).max(0), np.abs(W).max(0)
    T_x, T_w = float(np.float32(np.median(cx) * 1.5)), float(np.float32(np.median(cw) * 1.5))
    src, rx, rw, od, kp, kpad = O.plan_xw(cx, T_x, cw, T_w)
    assert kp == int(sum(max(1, np.ceil(float(a) / T_x)) * max(1, np.ceil(float(b) / T_w)) for a, b in zip(cx, cw)))
    Xf, Wf = O.flatten_float(X, src, rx), O.flatten_float(W, src, rw)
    ref = X.astype(np.float64) @ W.astype(np.float64).T
    np.testing.assert_allclose(Xf @ Wf.T, ref, rtol=1e-11, atol=1e-11 * np.abs(ref).max())
    assert np.abs(Xf).max() <= T_x and np.abs(Wf).max() <= T_w
    assert (rw > 1).any() and (rx > 1).any()


def test_flatten_weights_split_hand_case_and_reduction():
    # channel 1 of W exceeds T_w = 1 twice over: two shares of w/2; a_w = 1; qmax/a_w = 127, 63.5 on the shares
    W = np.array([[0.5, -1.0], [0.25, 2.0]], dtype=np.float32)
    src, rx, rw, od, kp, kpad = O.plan_xw([0.1, 0.1], 1.0, [0.5, 2.0], 1.0, align=1)
    assert src.tolist() == [0, 1, 1] and rw.tolist() == [1, 2, 2]
    Wq, s_w = O.flatten_weights_split(W, src, rw, 8)
    assert Wq.tolist() == [[64, -64, -64], [32, 127, 127]]          # 63.5 and -63.5 round to even
    assert s_w == np.float32(1.0 / 127.0)
    # with no weight channel split it is the plain quantize-and-repeat
    rng = np.random.default_rng(5)
    W = rng.standard_normal((6, 20)).astype(np.float32)
    src, rep, kp, kpad = O.plan(np.abs(rng.standard_normal(20) * 3).astype(np.float32), 2.0)
    ones = np.where(src >= 0, 1, 0).astype(np.int32)
    for bits in (8, 4):
        a, sa = O.flatten_weights_split(W, src, ones, bits)
        b, sb = O.flatten_weights(W, src, bits)
        np.testing.assert_array_equal(a, b)
        assert sa == sb


def test_peel_quantized_hand_case():
    """T = 2, x = 5 -> [2, 2, 1]; x = -3 -> [-2, -1]; x = 0.5 -> [0.5].  a' = T: m = 63.5 (INT8), 3.5 (INT4)."""
    X = np.array([[5.0, -3.0, 0.5]], dtype=np.float32)
    src, rx, rw, od, kp, kpad = O.plan_xw([5, 3, 0.5], 2.0, align=1)
    assert src.tolist() == [0, 1, 2, 0, 0, 1] and od.tolist() == [0, 0, 0, 1, 2, 1]
    q8, s8 = O.flatten_quant_act_peel(X, src, od, 8, 2.0, 2.0)
    assert q8.tolist() == [[127, -127, 32, 127, 64, -64]]           # 31.75 -> 32, 63.5 -> 64, -63.5 -> -64
    assert s8 == np.float32(2.0 / 127.0)
    q4, s4 = O.flatten_quant_act_peel(X, src, od, 4, 2.0, 2.0)
    assert q4.tolist() == [[7, -7, 2, 7, 4, -4]]                    # 1.75 -> 2, 3.5 -> 4 (even)
    assert s4 == np.float32(2.0 / 7.0)
    assert O.act_absmax_peel(X, 2.0) == np.float32(2.0)
    assert O.act_absmax_peel(X * 0.1, 2.0) == np.float32(0.5)
    qz, sz = O.flatten_quant_act_peel(X, src, od, 8, 2.0, 0.0)
    assert not qz.any() and sz == np.float32(1.0)


@pytest.mark.parametrize("bits", [8, 4])
def test_peel_quantized_against_the_float_split_and_reconstruction(bits):
    rng = np.random.default_rng(77)
    M, K = 31, 64
    X = (rng.standard_normal((M, K)) * rng.choice([1, 1, 1, 15], K)).astype(np.float32)
    ch = np.abs(X).max(0)
    T = float(np.float32(np.median(ch) * 1.2))
    src, rx, rw, od, kp, kpad = O.plan_xw(ch, T)
    q, s_x = O.flatten_quant_act_peel(X, src, od, bits, T, T)
    qmax = 2 ** (bits - 1) - 1
    # against the float64 split of the same equation, quantized in float64: equal except at fp32-vs-fp64 ties
    want = np.clip(np.rint(O.flatten_float_peel(X, src, T) * (qmax / T)), -qmax - 1, qmax)
    diff = np.abs(q.astype(np.int64) - want.astype(np.int64))
    assert diff.max() <= 1 and (diff != 0).mean() < 0.01
    # each slot is within half a step of its share, so a channel's slots sum back to x within n/2 steps
    recon = np.zeros((M, K))
    np.add.at(recon, (slice(None), src[:kp]), q[:, :kp].astype(np.float64) * float(s_x))
    n = rx[:K].astype(np.float64)
    assert (np.abs(recon - X) <= 0.5 * float(s_x) * n + 1e-6).all()
    assert not q[:, kp:].any()
    # full slots saturate at qmax: an element above 2T has its first two slots at +-qmax
    i, j = np.unravel_index(np.argmax(np.abs(X)), X.shape)
    slots = np.flatnonzero(src == j)
    assert abs(int(q[i, slots[0]])) == qmax and abs(int(q[i, slots[1]])) == qmax
