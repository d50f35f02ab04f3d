"""Pins for the oracle's integer GEMM, dequantization and the method's losslessness identity
(arXiv 2402.17985 Sec. 4.1: flatten + repeat "does not result in any precision loss";
Eq. 1 inverse for the dequantization)."""
import numpy as np
import pytest

import fq_workloads as WL
from oracle import fq_oracle as O


def test_gemm_hand_case():
    Xq = np.array([[1, -2, 3, 0], [127, 127, -128, 5]], np.int8)
    Wq = np.array([[4, 5, -6, 9], [-128, 127, 1, 0], [0, 0, 0, 0]], np.int8)
    # row 0: 4-10-18+0 = -24 ; -128-254+3 = -379 ; 0
    # row 1: 508+635+768+45 = 1956 ; -16256+16129-128+0 = -255 ; 0
    assert O.gemm_i32(Xq, Wq).tolist() == [[-24, -379, 0], [1956, -255, 0]]
    assert O.dot_i32(Xq[1], Wq[0]) == 1956


@pytest.mark.parametrize("seed,M,N,Kp", [(0, 3, 5, 32), (1, 7, 4, 96), (2, 1, 1, 64)])
def test_gemm_brute_force_python_ints(seed, M, N, Kp):
    rng = np.random.default_rng(seed)
    Xq = rng.integers(-128, 128, (M, Kp), dtype=np.int8)
    Wq = rng.integers(-128, 128, (N, Kp), dtype=np.int8)
    acc = O.gemm_i32(Xq, Wq)
    for i in range(M):
        for n in range(N):
            assert int(acc[i, n]) == sum(int(Xq[i, p]) * int(Wq[n, p]) for p in range(Kp))


def test_gemm_against_int64_library_matmul_and_row_window():
    rng = np.random.default_rng(7)
    M, N, Kp = 70, 45, 352
    Xq = rng.integers(-128, 128, (M, Kp), dtype=np.int8)
    Wq = rng.integers(-128, 128, (N, Kp), dtype=np.int8)
    ref = Xq.astype(np.int64) @ Wq.astype(np.int64).T
    assert (O.gemm_i32(Xq, Wq) == ref).all()
    assert (O.gemm_i32(Xq, Wq, row0=13, rows=20) == ref[13:33]).all()
    # transposed operand would be caught: the result is not symmetric in its operands
    assert not np.array_equal(O.gemm_i32(Xq[:45], Wq), O.gemm_i32(Wq, Xq[:45]))
    # the sum does not depend on the order of the flattened channels
    perm = rng.permutation(Kp)
    assert (O.gemm_i32(Xq[:, perm], Wq[:, perm]) == ref).all()


def test_extreme_values_accumulate_without_wrap():
    Kp = 26016                                  # largest flattened width among the workloads
    Xq = np.full((1, Kp), -128, np.int8)
    Wq = np.full((2, Kp), -128, np.int8)
    Wq[1] = 127
    assert O.gemm_i32(Xq, Wq).tolist() == [[Kp * 16384, -Kp * 16256]]


def test_dequant_closed_form():
    acc = np.array([[0, 1, -3, 2**31 - 1, -2**31]], np.int32)
    s_x, s_w = np.float32(0.015748031), np.float32(0.0078125)
    y = O.dequant(acc, s_x, s_w)
    for a, v in zip(acc[0], y[0]):
        assert v == float(int(a)) * float(s_x) * float(s_w)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_flatten_repeat_is_lossless_in_float64(seed):
    """X'W' = XW (Sec. 4.1) and max|x'| <= T, for the equal split and for the printed peel split."""
    rng = np.random.default_rng(seed)
    M, K, N = 24, 80, 17
    X = rng.standard_normal((M, K)).astype(np.float32)
    X[:, rng.choice(K, 5, replace=False)] *= rng.uniform(10, 100, 5).astype(np.float32)
    W = (rng.standard_normal((N, K)) / np.sqrt(K)).astype(np.float32)
    chmax = np.abs(X).max(axis=0)
    T = float(np.float32(1.3 * np.median(chmax)))
    src, rep, kp, kpad = O.plan(chmax, T, 32)
    assert kp > K
    ref = X.astype(np.float64) @ W.astype(np.float64).T            # library float64 product
    np.testing.assert_allclose(O.linear_f64(X, W), ref, rtol=1e-12, atol=1e-13)
    Wf = O.repeat_weights_float(W, src)
    for Xf in (O.flatten_float(X, src, rep), O.flatten_float_peel(X, src, T)):
        assert np.abs(Xf).max() <= T
        got = O.matmul_nt_f64(Xf, Wf)
        np.testing.assert_allclose(got, ref, rtol=1e-11, atol=1e-12)
        np.testing.assert_allclose(Xf @ Wf.T, ref, rtol=1e-11, atol=1e-12)


def test_copies_contribute_n_times_in_the_integer_product():
    """A channel with n copies contributes n * q(x/n) * q(w) to the accumulator (Eq. 3-4)."""
    X = np.array([[0.5, 9.0], [1.0, -4.5]], np.float32)
    W = np.array([[1.0, -0.5]], np.float32)
    chmax = np.abs(X).max(axis=0)
    src, rep, kp, kpad = O.plan(chmax, 3.0, 32)           # channel 1: n = 3
    assert rep[1] == 3
    Wq, s_w = O.flatten_weights(W, src, 8)
    a = O.act_absmax_dynamic(X, src, rep)                  # = 3.0
    Xq, s_x = O.flatten_quant_act(X, src, rep, 8, a)
    acc = O.gemm_i32(Xq, Wq)
    for i in range(2):
        assert acc[i, 0] == int(Xq[i, 0]) * int(Wq[0, 0]) + 3 * int(Xq[i, 1]) * int(Wq[0, 1])
    # by hand: 1/s_x = 127/3; row 0: q(0.5) = rne(21.17) = 21, q(9/3) = 127; W: 127, -64 (tie -63.5 -> -64)
    assert Xq[0, :2].tolist() == [21, 127] and Wq[0, :2].tolist() == [127, -64]
    assert acc[0, 0] == 21 * 127 + 3 * 127 * -64


@pytest.mark.parametrize("bits", [8, 4])
def test_whole_layer_equals_its_steps_and_tracks_the_float_product(bits):
    L = WL.make_layer(WL.CONFIGS["cfg1b"], 0)
    src, rep, kp, kpad = O.plan(L.chmax, L.T)
    Wq, s_w = O.flatten_weights(L.W, src, bits)
    acc, y, s_x = O.linear(L.X, src, rep, Wq, s_w, bits)
    a = O.act_absmax_dynamic(L.X, src, rep)
    Xq, s_x2 = O.flatten_quant_act(L.X, src, rep, bits, a)
    assert s_x == s_x2
    assert (acc == Xq.astype(np.int64) @ Wq.astype(np.int64).T).all()
    assert (y == acc.astype(np.float64) * float(s_x) * float(s_w)).all()
    ref = L.X.astype(np.float64) @ L.W.astype(np.float64).T
    rel = np.linalg.norm(y - ref) / np.linalg.norm(ref)
    assert rel < (0.02 if bits == 8 else 0.3)
    # a row window with the per-tensor scale taken over all rows
    acc_w, y_w, s_x_w = O.linear(L.X, src, rep, Wq, s_w, bits, row0=5, rows=4)
    assert s_x_w == s_x and (acc_w == acc[5:9]).all()


def test_error_shrinks_as_threshold_shrinks():
    """The paper's accuracy argument in miniature (Sec. 4.1-4.2): a lower truncation threshold
    gives a finer per-tensor grid, so the INT8 layer output approaches the float product."""
    L = WL.make_layer(WL.CONFIGS["cfg2"], 0, M_override=64, K_override=512, N_override=48)
    ref = L.X.astype(np.float64) @ L.W.astype(np.float64).T
    errs = []
    for T in (float(L.chmax.max()), float(L.chmax.max()) / 8, float(np.median(L.chmax)) * 2):
        src, rep, kp, kpad = O.plan(L.chmax, T)
        Wq, s_w = O.flatten_weights(L.W, src, 8)
        _, y, _ = O.linear(L.X, src, rep, Wq, s_w, 8)
        errs.append(np.linalg.norm(y - ref) / np.linalg.norm(ref))
    assert errs[0] > errs[1] > errs[2]


def test_bmm_hand_case_and_library():
    """Batched product (Sec. 5.1): a hand case with distinct batches (a swapped batch index, a
    transposed operand or a dropped term changes it), NumPy's int64 einsum, and batch = 1 against
    the plain GEMM."""
    A = np.array([[[1, 2], [3, 4], [-1, 0]], [[0, 1], [5, -6], [7, 7]]], dtype=np.int8)      # [2, 3, 2]
    B = np.array([[[1, 0], [2, -1]], [[-3, 1], [1, 1]]], dtype=np.int8)                      # [2, 2, 2]
    want = [[[1, 0], [3, 2], [-1, -2]], [[1, 1], [-21, -1], [-14, 14]]]
    assert O.bmm_i32(A, B).tolist() == want
    rng = np.random.default_rng(11)
    A = rng.integers(-128, 128, (5, 17, 96), dtype=np.int8)
    B = rng.integers(-128, 128, (5, 9, 96), dtype=np.int8)
    ref = np.einsum("bik,bnk->bin", A.astype(np.int64), B.astype(np.int64))
    got = O.bmm_i32(A, B)
    np.testing.assert_array_equal(got, ref)
    np.testing.assert_array_equal(O.bmm_i32(A[2:3], B[2:3])[0], O.gemm_i32(A[2], B[2]))


def test_dequant_bias_hand_case():
    """y = acc * s_x * s_w + bias[n]: exact binary fractions, so the float64 result is exact; the bias
    goes with the column (a row/column mix-up changes the values)."""
    acc = np.array([[4, -8, 0], [2, 2, 2]], dtype=np.int32)
    y = O.dequant_bias(acc, np.float32(0.5), np.float32(0.25), np.array([1.0, -2.0, 0.5], np.float32))
    assert y.tolist() == [[1.5, -3.0, 0.5], [1.25, -1.75, 0.75]]
    np.testing.assert_array_equal(O.dequant_bias(acc, np.float32(0.3), np.float32(0.7), np.zeros(3, np.float32)),
                                  O.dequant(acc, np.float32(0.3), np.float32(0.7)))
