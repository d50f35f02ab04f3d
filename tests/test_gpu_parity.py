"""GPU parity: every call of the C ABI against the CPU oracle on the same seeded inputs.

Bars (arXiv 2402.17985 fixes the arithmetic; the tolerances follow from it):
  - flatten maps, quantized INT8 / packed INT4 tensors, scales and int32 accumulators: bit-exact;
  - dequantized outputs: the stored fp32 / half / bfloat16 bit patterns equal the oracle's rounded output
    fl32(fl32(acc) * fl32(s_x * s_w)) (+ bias), rounded to nearest-even to the output type: bit-exact;
  - and, as a sanity line, against the oracle's unrounded float64 y = acc * s_x * s_w:
      fp32 out  <= 1e-6 relative  (fl32(acc), fl32(s_x*s_w) and one multiply: 3 roundings of 2^-24),
      fp16 out  <= 1e-3 relative  (half ulp 4.9e-4 on top of the above),
      bf16 out  <= 2^-8 relative  (bf16 keeps 8 significand bits: its own rounding is up to 2^-9;
                 the fp32 value before that rounding is held to 1e-6 by the fp32 case).
"""
import numpy as np
import pytest
import torch

import fq_workloads as WL
import paper_2402_17985_amd as fq
from oracle import fq_oracle as O
from tests.gpu_util import DEV, bf16_to_f64, bits16, bits32, bytes_ws, dev_i32, rel_err, scalar, to_dev

pytestmark = pytest.mark.gpu


def _layer(cfg, idx=0, **over):
    return WL.make_layer(WL.CONFIGS[cfg], idx, **over)


def _gpu_flatten_quant(L, src, rep, bits, a_static=None, X_dev=None):
    M, K = L.X.shape
    Kpad = len(src)
    Xd = to_dev(L.X_store, L.spec.x_dtype) if X_dev is None else X_dev
    out = torch.full((M, Kpad if bits == 8 else Kpad // 2), 0x55, dtype=torch.uint8, device=DEV)
    s_x = torch.zeros(1, dtype=torch.float32, device=DEV)
    ws = bytes_ws(fq.fq_act_workspace_bytes(K, Kpad))
    fq.fq_flatten_quant_act(Xd, dev_i32(src), dev_i32(rep), bits, out, s_x, ws,
                            absmax_in=None if a_static is None else scalar(a_static))
    torch.cuda.synchronize()
    return out.cpu().numpy(), np.float32(s_x.item())


def _oracle_flatten_quant(L, src, rep, bits, a_static=None):
    a = O.act_absmax_dynamic(L.X, src, rep) if a_static is None else np.float32(a_static)
    q, s_x = O.flatten_quant_act(L.X, src, rep, bits, a)
    return (q.view(np.uint8) if bits == 8 else O.pack_i4(q)), s_x


# ------------------------------------------------------------------------------------------
# flatten + quantize (activations)
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("cfg,over", [
    ("cfg1", {}), ("cfg1b", {}),
    ("cfg2", dict(M_override=333, K_override=1000, N_override=8)),        # ragged M, K not a multiple of 16
    ("cfg3", dict(M_override=517, K_override=2048, N_override=8)),
    ("cfg4", dict(M_override=70, K_override=5120, N_override=8)),
])
def test_flatten_quant_act_dynamic(cfg, over, bits):
    L = _layer(cfg, **over)
    if L.spec.x_dtype != "f32" and L.X.shape[1] % 8:
        pytest.skip("row stride must be a multiple of 16 bytes")
    src, rep, kp, kpad = fq.fq_flatten_plan(L.chmax, L.T)
    osrc, orep, okp, okpad = O.plan(L.chmax, L.T)
    assert (kp, kpad) == (okp, okpad) and (src == osrc).all() and (rep == orep).all()
    got, s_x = _gpu_flatten_quant(L, src, rep, bits)
    want, s_x_o = _oracle_flatten_quant(L, src, rep, bits)
    assert s_x == s_x_o
    assert np.array_equal(got, want)


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_flatten_quant_act_static_clamps_and_dtypes(bits, dtype):
    """The paper's static mode with a' = T; chmax is deliberately understated for two channels so
    that values beyond the calibrated range reach the clamp."""
    rng = np.random.default_rng(11)
    M, K = 129, 264
    X = rng.standard_normal((M, K), dtype=np.float32)
    X[:, [5, 77, 200]] *= np.array([30, 12, 55], np.float32)
    store, Xf = WL.round_to_dtype(X, dtype)
    chmax = np.abs(Xf).max(axis=0)
    chmax[[5, 100]] *= 0.5
    T = 2.0
    src, rep, kp, kpad = fq.fq_flatten_plan(chmax, T)
    L = WL.Layer(WL.LayerSpec("s", M, K, 8, bits, dtype, dtype), store, Xf, None, None, chmax, T)
    got, s_x = _gpu_flatten_quant(L, src, rep, bits, a_static=T)
    want, s_x_o = _oracle_flatten_quant(L, src, rep, bits, a_static=T)
    assert s_x == s_x_o and np.array_equal(got, want)
    q = want.view(np.int8) if bits == 8 else O.unpack_i4(want)
    assert q.min() == -(1 << (bits - 1))                     # the clamp is live


def test_flatten_quant_act_strided_rows_zero_input_and_bad_map():
    rng = np.random.default_rng(3)
    M, K, ld = 40, 96, 128
    buf = torch.zeros((M, ld), dtype=torch.float32, device=DEV)
    X = rng.standard_normal((M, K), dtype=np.float32)
    X[:, 9] *= 25
    buf[:, :K] = torch.from_numpy(X).to(DEV)
    chmax = np.abs(X).max(axis=0)
    src, rep, kp, kpad = fq.fq_flatten_plan(chmax, 3.0)
    L = WL.Layer(WL.LayerSpec("s", M, K, 8, 8, "f32", "f32"), X, X, None, None, chmax, 3.0)
    got, s_x = _gpu_flatten_quant(L, src, rep, 8, X_dev=buf[:, :K])
    want, s_x_o = _oracle_flatten_quant(L, src, rep, 8)
    assert s_x == s_x_o and np.array_equal(got, want)
    # all-zero activations: zeros out, s_x = 1
    Lz = WL.Layer(L.spec, np.zeros_like(X), np.zeros_like(X), None, None, chmax, 3.0)
    got, s_x = _gpu_flatten_quant(Lz, src, rep, 8)
    assert s_x == np.float32(1.0) and not got.any()
    # a map with out-of-range sources: those slots read as padding, nothing faults
    bad = src.copy()
    bad[3] = K + 1000
    bad[kp - 1] = -7
    got, _ = _gpu_flatten_quant(L, bad, rep, 8)
    good = src.copy()
    good[3] = -1
    good[kp - 1] = -1
    want, _ = _oracle_flatten_quant(L, good, rep, 8)
    assert np.array_equal(got, want)


def _synthetic_layer(seed, M, K, dtype, n_out, factor, T_mult):
    """A layer's activation side built directly (shapes the workload table has no entry for)."""
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((M, K), dtype=np.float32)
    idx = rng.choice(K, n_out, replace=False)
    X[:, idx] *= np.float32(factor)
    store, Xf = WL.round_to_dtype(X, dtype)
    chmax = np.abs(Xf).max(axis=0).astype(np.float32)
    T = float(np.float32(T_mult * np.median(chmax)))
    return WL.Layer(WL.LayerSpec("synthetic", M, K, 8, 8, dtype, dtype), store, Xf, None, None, chmax, T)


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("K,n_out", [(8, 1), (66000, 40)])
def test_flatten_quant_act_general_kernel_narrow_and_very_wide(K, n_out, bits):
    """K < 16 and a layer too wide for the row-strip kernel's LDS budget: the equal split through the general
    one-thread-per-16-slots kernel, dynamic scale, byte for byte."""
    L = _synthetic_layer(40 + K % 7, 4, K, "bf16", n_out, 30.0, 3.0)
    src, rep, kp, kpad = fq.fq_flatten_plan(L.chmax, L.T)
    assert kpad > K and kpad < 131072
    got, s_x = _gpu_flatten_quant(L, src, rep, bits)
    want, s_x_o = _oracle_flatten_quant(L, src, rep, bits)
    assert s_x == s_x_o
    assert np.array_equal(got, want)


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("dtype,K,ld", [("bf16", 1004, 1008), ("f32", 202, 204), ("f16", 1004, 1008)])
def test_flatten_quant_act_ragged_last_column_group(dtype, K, ld, bits):
    """K not a multiple of the 16-byte vector width with an aligned row stride: the absmax kernel's last column
    group is read element by element.  The outliers sit in that ragged tail so that it decides the scale."""
    rng = np.random.default_rng(50 + K)
    M = 300
    X = rng.standard_normal((M, K), dtype=np.float32)
    X[:, K - 1] *= 40.0
    X[:, K - 3] *= 17.0
    store, Xf = WL.round_to_dtype(X, dtype)
    chmax = np.abs(Xf).max(axis=0).astype(np.float32)
    T = float(np.float32(3.0 * np.median(chmax)))
    L = WL.Layer(WL.LayerSpec("ragged", M, K, 8, 8, dtype, dtype), store, Xf, None, None, chmax, T)
    tdt = {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32}[dtype]
    buf = torch.zeros((M, ld), dtype=tdt, device=DEV)
    buf[:, :K] = to_dev(store, dtype)
    src, rep, kp, kpad = fq.fq_flatten_plan(chmax, T)
    got, s_x = _gpu_flatten_quant(L, src, rep, bits, X_dev=buf[:, :K])
    want, s_x_o = _oracle_flatten_quant(L, src, rep, bits)
    assert s_x == s_x_o
    assert np.array_equal(got, want)


# ------------------------------------------------------------------------------------------
# weights (offline)
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("cfg,over", [("cfg1b", {}), ("cfg2", dict(M_override=64, K_override=1024, N_override=301))])
def test_flatten_weights(cfg, over, bits):
    L = _layer(cfg, **over)
    Wd = to_dev(L.W_store, L.spec.w_dtype)
    lay = fq.FqLinear(Wd, L.chmax, L.T, bits)
    torch.cuda.synchronize()
    align = 128 if bits == 8 else 256                      # the layer's default row alignment
    src, rep, kp, kpad = O.plan(L.chmax, L.T, align)
    assert (lay.src_host == src).all() and (lay.rep_host == rep).all() and lay.Kpad == kpad
    Wq_o, s_w_o = O.flatten_weights(L.W, src, bits)
    want = Wq_o.view(np.uint8) if bits == 8 else O.pack_i4(Wq_o)
    assert np.float32(lay.s_w.item()) == s_w_o
    assert np.array_equal(lay.Wq.cpu().numpy().view(np.uint8), want)


# ------------------------------------------------------------------------------------------
# integer GEMM: raw accumulators, every tile variant, ragged shapes
# ------------------------------------------------------------------------------------------
def _rand_q(rng, rows, Kpad, bits):
    lo, hi = -(1 << (bits - 1)), (1 << (bits - 1))
    return rng.integers(lo, hi, (rows, Kpad), dtype=np.int8)


def _gemm_acc(Xq, Wq, bits):
    M, N = Xq.shape[0], Wq.shape[0]
    Y = torch.full((M, N), -12345, dtype=torch.int32, device=DEV)
    if bits == 8:
        fq.fq_gemm_i8(torch.from_numpy(Xq).to(DEV), torch.from_numpy(Wq).to(DEV), None, None, Y)
    else:
        fq.fq_gemm_i4(torch.from_numpy(O.pack_i4(Xq)).to(DEV), torch.from_numpy(O.pack_i4(Wq)).to(DEV), None, None, Y)
    torch.cuda.synchronize()
    return Y.cpu().numpy()


@pytest.mark.parametrize("variant", [2, 6, 7, 10])
@pytest.mark.parametrize("bits", [8, 4])
def test_gemm_accumulators_bit_exact(variant, bits):
    rng = np.random.default_rng(100 * variant + bits)
    fq.fq_gemm_select(variant)
    try:
        # several tiles + ragged tails in M and N; Kpad = 32 mod 64 / 128 exercises the masked last k-stage
        for (M, N, Kpad) in [(300, 520, 416), (257, 129, 1056), (1, 1, 32), (33, 700, 160)]:
            Xq, Wq = _rand_q(rng, M, Kpad, bits), _rand_q(rng, N, Kpad, bits)
            got = _gemm_acc(Xq, Wq, bits)
            assert np.array_equal(got, O.gemm_i32(Xq, Wq)), (variant, bits, M, N, Kpad)
    finally:
        fq.fq_gemm_select(-1)


@pytest.mark.parametrize("bits", [8, 4])
def test_gemm_extreme_values_do_not_wrap(bits):
    Kpad, lo = 26016, -(1 << (bits - 1))
    Xq = np.full((40, Kpad), lo, np.int8)
    Wq = np.full((70, Kpad), lo, np.int8)
    Wq[1::2] = -lo - 1
    got = _gemm_acc(Xq, Wq, bits)
    assert np.array_equal(got, O.gemm_i32(Xq, Wq))
    assert got[0, 0] == Kpad * lo * lo


@pytest.mark.parametrize("ydt,tol", [(torch.float32, 1e-6), (torch.float16, 1e-3), (torch.bfloat16, 2.0 ** -8)])
def test_gemm_dequant_epilogue(ydt, tol):
    rng = np.random.default_rng(5)
    M, N, Kpad = 200, 333, 512
    Xq, Wq = _rand_q(rng, M, Kpad, 8), _rand_q(rng, N, Kpad, 8)
    s_x, s_w = np.float32(0.0123), np.float32(0.00071)
    ldy = 336
    Ybuf = torch.full((M, ldy), 7.0, dtype=ydt, device=DEV)
    fq.fq_gemm_i8(torch.from_numpy(Xq).to(DEV), torch.from_numpy(Wq).to(DEV), scalar(s_x), scalar(s_w), Ybuf[:, :N])
    torch.cuda.synchronize()
    ref = O.dequant(O.gemm_i32(Xq, Wq), s_x, s_w)
    got = Ybuf[:, :N].float().cpu().numpy().astype(np.float64)
    assert rel_err(got, ref).max() <= tol
    assert (Ybuf[:, N:].float() == 7.0).all()                # nothing written beyond column N
    # the stored bit patterns are the oracle's rounded output
    name = {torch.float32: "f32", torch.float16: "f16", torch.bfloat16: "bf16"}[ydt]
    exact = O.dequant_out(O.gemm_i32(Xq, Wq), s_x, s_w, name)
    stored = bits32(Ybuf[:, :N]) if ydt == torch.float32 else bits16(Ybuf[:, :N])
    assert np.array_equal(stored, exact.view(np.uint32) if ydt == torch.float32 else exact)


# ------------------------------------------------------------------------------------------
# the whole layer
# ------------------------------------------------------------------------------------------
def _run_linear(L, bits, ydt, a_static=None):
    Wd = to_dev(L.W_store, L.spec.w_dtype)
    lay = fq.FqLinear(Wd, L.chmax, L.T, bits)
    Xd = to_dev(L.X_store, L.spec.x_dtype)
    Y = lay.forward(Xd, out_dtype=ydt, absmax_in=None if a_static is None else scalar(a_static))
    torch.cuda.synchronize()
    return lay, Y


@pytest.mark.parametrize("cfg,over,bits", [
    ("cfg1", {}, 8), ("cfg1b", {}, 8), ("cfg1b", {}, 4),
    ("cfg2", dict(M_override=300, K_override=1024, N_override=520), 8),
    ("cfg3", dict(M_override=384, K_override=1024, N_override=700), 4),
    ("cfg4", dict(M_override=260, K_override=2048, N_override=264), 4),
])
def test_linear_end_to_end(cfg, over, bits):
    L = _layer(cfg, **over)
    src, rep, kp, kpad = O.plan(L.chmax, L.T, 128 if bits == 8 else 256)
    Wq_o, s_w_o = O.flatten_weights(L.W, src, bits)
    acc_o, y_o, s_x_o = O.linear(L.X, src, rep, Wq_o, s_w_o, bits)
    lay, acc = _run_linear(L, bits, torch.int32)
    assert (lay.src_host == src).all() and (lay.rep_host == rep).all()
    assert np.array_equal(acc.cpu().numpy(), acc_o)
    _, y32 = _run_linear(L, bits, torch.float32)
    assert rel_err(y32.cpu().numpy().astype(np.float64), y_o).max() <= 1e-6
    _, y16 = _run_linear(L, bits, torch.bfloat16)
    assert rel_err(bf16_to_f64(y16), y_o).max() <= 2.0 ** -8
    # static mode (the paper's): a' = T
    acc_s, _, _ = O.linear(L.X, src, rep, Wq_o, s_w_o, bits, a_static=L.T)
    _, acc_sg = _run_linear(L, bits, torch.int32, a_static=L.T)
    assert np.array_equal(acc_sg.cpu().numpy(), acc_s)


def test_linear_is_deterministic():
    L = _layer("cfg2", M_override=512, K_override=1024, N_override=512)
    lay, a = _run_linear(L, 8, torch.bfloat16)
    Xd = to_dev(L.X_store, L.spec.x_dtype)
    b = lay.forward(Xd, out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))


# ------------------------------------------------------------------------------------------
# bf16 baseline GEMM
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("variant,K", [(7, 1032), (2, 1032), (11, 1024), (11, 192), (12, 1024), (12, 192), (12, 64), (12, 128)])
def test_gemm_bf16_baseline(variant, K):
    rng = np.random.default_rng(9)
    M, N = 300, 260
    Xs, Xf = WL.round_to_dtype(rng.standard_normal((M, K), dtype=np.float32), "bf16")
    Ws, Wf = WL.round_to_dtype(rng.standard_normal((N, K), dtype=np.float32) / np.float32(np.sqrt(K)), "bf16")
    Y = torch.zeros((M, N), dtype=torch.bfloat16, device=DEV)
    fq.fq_gemm_select(variant)
    try:
        fq.fq_gemm_bf16(to_dev(Xs, "bf16"), to_dev(Ws, "bf16"), Y)
        torch.cuda.synchronize()
    finally:
        fq.fq_gemm_select(-1)
    ref = Xf.astype(np.float64) @ Wf.astype(np.float64).T
    # fp32 accumulation of K products, then one bf16 rounding
    assert rel_err(bf16_to_f64(Y), ref).max() <= 2.0 ** -8 + 1e-4


def test_gemm_bf16_baseline_large_default():
    """A problem large enough (210 tiles of 256 x 256, ragged edges, half-height tail) for the automatic choice
    to take the large-problem kernel; sampled rows against the float64 product."""
    rng = np.random.default_rng(10)
    M, N, K = 15 * 256 - 30, 14 * 256 - 9, 256
    Xs, Xf = WL.round_to_dtype(rng.standard_normal((M, K), dtype=np.float32), "bf16")
    Ws, Wf = WL.round_to_dtype(rng.standard_normal((N, K), dtype=np.float32) / np.float32(np.sqrt(K)), "bf16")
    Y = torch.zeros((M, N + 1), dtype=torch.bfloat16, device=DEV)
    fq.fq_gemm_bf16(to_dev(Xs, "bf16"), to_dev(Ws, "bf16"), Y[:, :N])
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([rng.integers(0, M, 60), [0, M - 1, 255, 256, 3583, 3584]]))
    ref = Xf[rows].astype(np.float64) @ Wf.astype(np.float64).T
    assert rel_err(bf16_to_f64(Y[torch.from_numpy(rows).to(DEV)][:, :N]), ref).max() <= 2.0 ** -8 + 1e-4
    assert not Y[:, N:].any()


# ------------------------------------------------------------------------------------------
# calibration statistic and the paper's threshold rule on top of it
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("cfg,over", [
    ("cfg1", {}),
    ("cfg2", dict(M_override=333, K_override=1000, N_override=8)),
    ("cfg3", dict(M_override=1100, K_override=4096, N_override=8)),
    ("cfg4", dict(M_override=70, K_override=5120, N_override=8)),
])
def test_channel_absmax_and_boxplot_threshold(cfg, over):
    """fq_channel_absmax bit-exact against the oracle (one batch, then a second batch accumulated),
    and Eq. 6-7 on its result gives the oracle's threshold and plan."""
    L = _layer(cfg, **over)
    if L.spec.x_dtype != "f32" and L.X.shape[1] % 8:
        pytest.skip("row stride must be a multiple of 16 bytes")
    M, K = L.X.shape
    Xd = to_dev(L.X_store, L.spec.x_dtype)
    ch = torch.full((K,), 123.0, dtype=torch.float32, device=DEV)       # stale contents must be overwritten
    half = max(1, M // 2)
    fq.fq_channel_absmax(Xd[:half], ch)
    torch.cuda.synchronize()
    ref1 = O.channel_absmax(L.X[:half])
    np.testing.assert_array_equal(ch.cpu().numpy(), ref1)
    if half < M:
        fq.fq_channel_absmax(Xd[half:], ch, accumulate=True)
        torch.cuda.synchronize()
    ref = O.channel_absmax(L.X[half:], prev=ref1) if half < M else ref1
    got = ch.cpu().numpy()
    np.testing.assert_array_equal(got, ref)
    np.testing.assert_array_equal(ref, np.abs(L.X).max(axis=0))
    T = fq.fq_threshold_boxplot(got, 1.3)
    T_ref = float(O.threshold_boxplot(ref, 1.3))
    assert abs(T - T_ref) <= 1e-6 * T_ref
    src, rep, kp, kpad = fq.fq_flatten_plan(got, T_ref)
    src_o, rep_o, kp_o, kpad_o = O.plan(ref, T_ref)
    assert (kp, kpad) == (kp_o, kpad_o)
    np.testing.assert_array_equal(src, src_o)
    np.testing.assert_array_equal(rep, rep_o)


# ------------------------------------------------------------------------------------------
# batched integer product (attention-shaped)
# ------------------------------------------------------------------------------------------
def _bmm_operands(seed, batch, M, N, Kpad, bits):
    rng = np.random.default_rng([seed, batch, M, N, Kpad, bits])
    lo, hi = (-128, 128) if bits == 8 else (-8, 8)
    A = rng.integers(lo, hi, (batch, M, Kpad), dtype=np.int8)
    B = rng.integers(lo, hi, (batch, N, Kpad), dtype=np.int8)
    return A, B


def _to_dev_q(q, bits):
    if bits == 8:
        return torch.from_numpy(q).to(DEV)
    b, r, k = q.shape
    return torch.from_numpy(O.pack_i4(q.reshape(b * r, k)).reshape(b, r, k // 2)).to(DEV)


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("batch,M,N,Kpad", [
    (3, 200, 200, 128),        # Q K^T shape: short reduction, ragged tiles
    (5, 257, 128, 320),        # P V shape: N = head size, reduction over the sequence
    (2, 64, 40, 32),           # tiny
    (1, 130, 300, 1024),       # batch of one equals the plain GEMM
    (7, 129, 131, 96),
])
def test_bmm_accumulators_bit_exact(batch, M, N, Kpad, bits):
    A, B = _bmm_operands(1, batch, M, N, Kpad, bits)
    ref = O.bmm_i32(A, B)
    Ad, Bd = _to_dev_q(A, bits), _to_dev_q(B, bits)
    Y = torch.full((batch, M, N), -7, dtype=torch.int32, device=DEV)
    (fq.fq_bmm_i8 if bits == 8 else fq.fq_bmm_i4)(Ad, Bd, None, None, Y)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(Y.cpu().numpy(), ref)


@pytest.mark.parametrize("variant", [2, 6, 7, 10])
def test_bmm_variants_and_padded_strides(variant):
    """Every kernel family with batch strides larger than one matrix (operands and output live in
    wider buffers; the gaps must stay untouched) and a 2-byte dequantized output."""
    batch, M, N, Kpad = 4, 300, 260, 256
    A, B = _bmm_operands(2, batch, M, N, Kpad, 8)
    ref = O.bmm_i32(A, B)
    Abuf = torch.zeros((batch, M + 5, Kpad), dtype=torch.int8, device=DEV)
    Bbuf = torch.zeros((batch, N + 3, Kpad), dtype=torch.int8, device=DEV)
    Abuf[:, :M] = torch.from_numpy(A).to(DEV)
    Bbuf[:, :N] = torch.from_numpy(B).to(DEV)
    s_a, s_b = scalar(0.013), scalar(0.0021)
    Ybuf = torch.full((batch, M + 2, N + 8), 99.0, dtype=torch.bfloat16, device=DEV)
    Yi = torch.zeros((batch, M, N), dtype=torch.int32, device=DEV)
    fq.fq_gemm_select(variant)
    try:
        fq.fq_bmm_i8(Abuf[:, :M], Bbuf[:, :N], s_a, s_b, Ybuf[:, :M, :N])
        fq.fq_bmm_i8(Abuf[:, :M], Bbuf[:, :N], None, None, Yi)
        torch.cuda.synchronize()
    finally:
        fq.fq_gemm_select(-1)
    np.testing.assert_array_equal(Yi.cpu().numpy(), ref)
    y_ref = O.dequant(ref, np.float32(0.013), np.float32(0.0021))
    got = bf16_to_f64(Ybuf[:, :M, :N])
    assert rel_err(got, y_ref).max() <= 2.0 ** -8
    full = Ybuf.float().cpu().numpy()
    assert (full[:, M:, :] == 99.0).all() and (full[:, :, N:] == 99.0).all()


# ------------------------------------------------------------------------------------------
# Eq. 3 as printed (peel split) and weight-side flattening
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("static", [False, True])
@pytest.mark.parametrize("cfg,over", [
    ("cfg1", {}),
    ("cfg2", dict(M_override=333, K_override=1000, N_override=8)),
    ("cfg3", dict(M_override=517, K_override=2048, N_override=8)),
])
def test_flatten_quant_act_peel(cfg, over, static, bits):
    L = _layer(cfg, **over)
    if L.spec.x_dtype != "f32" and L.X.shape[1] % 8:
        pytest.skip("row stride must be a multiple of 16 bytes")
    M, K = L.X.shape
    T = float(np.float32(L.T))
    src, rx, rw, od, kp, kpad = fq.fq_flatten_plan_xw(L.chmax, T)
    a_ref = np.float32(T) if static else O.act_absmax_peel(L.X, T)
    q_ref, s_ref = O.flatten_quant_act_peel(L.X, src, od, bits, T, a_ref)
    want = q_ref.view(np.uint8) if bits == 8 else O.pack_i4(q_ref)
    Xd = to_dev(L.X_store, L.spec.x_dtype)
    out = torch.full((M, kpad if bits == 8 else kpad // 2), 0x55, dtype=torch.uint8, device=DEV)
    s_x = torch.zeros(1, dtype=torch.float32, device=DEV)
    ws = bytes_ws(fq.fq_act_workspace_bytes(K, kpad))
    fq.fq_flatten_quant_act_peel(Xd, dev_i32(src), dev_i32(od), bits, T, out, s_x, ws,
                                 absmax_in=scalar(T) if static else None)
    torch.cuda.synchronize()
    assert np.float32(s_x.item()) == s_ref
    np.testing.assert_array_equal(out.cpu().numpy(), want)


@pytest.mark.parametrize("bits", [8, 4])
def test_two_sided_flatten_end_to_end(bits):
    """Weights' own channels split (fq_flatten_weights_split) together with the activation split over
    the two-sided map: quantized tensors and accumulators bit-exact, output close to the float layer."""
    L = _layer("cfg3", M_override=300, K_override=1024, N_override=200)
    M, K = L.X.shape
    N = L.W.shape[0]
    rng = np.random.default_rng(9)
    W = L.W.copy()
    W[:, rng.choice(K, 12, replace=False)] *= np.float32(5.0)               # a few large weight channels
    W_store, W = WL.round_to_dtype(W, L.spec.w_dtype)                       # 5x is exact only up to rounding
    cw = np.abs(W).max(axis=0)
    T_w = float(np.float32(2.0 * np.median(cw)))
    src, rx, rw, od, kp, kpad = fq.fq_flatten_plan_xw(L.chmax, float(L.T), cw, T_w, align=128 if bits == 8 else 256)
    assert (rw > 1).any() and (rx > 1).any()
    Wq_ref, s_w_ref = O.flatten_weights_split(W, src, rw, bits)
    Xq_ref, s_x_ref = O.flatten_quant_act(L.X, src, rx, bits, O.act_absmax_dynamic(L.X, src, rx))
    acc_ref = O.gemm_i32(Xq_ref, Wq_ref)
    cols = kpad if bits == 8 else kpad // 2
    Wd = to_dev(W_store, L.spec.w_dtype)
    Xd = to_dev(L.X_store, L.spec.x_dtype)
    Wq = torch.empty((N, cols), dtype=torch.uint8, device=DEV)
    Xq = torch.empty((M, cols), dtype=torch.uint8, device=DEV)
    s_w, s_x = scalar(0.0), scalar(0.0)
    ws = bytes_ws(fq.fq_act_workspace_bytes(K, kpad))
    srcd = dev_i32(src)
    fq.fq_flatten_weights_split(Wd, srcd, dev_i32(rw), bits, Wq, s_w, ws)
    fq.fq_flatten_quant_act(Xd, srcd, dev_i32(rx), bits, Xq, s_x, ws)
    acc = torch.empty((M, N), dtype=torch.int32, device=DEV)
    y = torch.empty((M, N), dtype=torch.float32, device=DEV)
    gemm = fq.fq_gemm_i8 if bits == 8 else fq.fq_gemm_i4
    Xv, Wv = (Xq.view(torch.int8), Wq.view(torch.int8)) if bits == 8 else (Xq, Wq)
    gemm(Xv, Wv, None, None, acc)
    gemm(Xv, Wv, s_x, s_w, y)
    torch.cuda.synchronize()
    assert np.float32(s_w.item()) == s_w_ref and np.float32(s_x.item()) == s_x_ref
    np.testing.assert_array_equal(Wq.cpu().numpy(), Wq_ref.view(np.uint8) if bits == 8 else O.pack_i4(Wq_ref))
    np.testing.assert_array_equal(Xq.cpu().numpy(), Xq_ref.view(np.uint8) if bits == 8 else O.pack_i4(Xq_ref))
    np.testing.assert_array_equal(acc.cpu().numpy(), acc_ref)
    y_ref = O.dequant(acc_ref, s_x_ref, s_w_ref)
    assert rel_err(y.cpu().numpy().astype(np.float64), y_ref).max() <= 1e-6
    # and the quantized layer tracks the float layer (INT8 closely, INT4 loosely)
    y_float = O.linear_f64(L.X, W)
    err = np.sqrt(np.mean((y_ref - y_float) ** 2)) / np.sqrt(np.mean(y_float ** 2))
    assert err < (0.03 if bits == 8 else 0.4)


# ------------------------------------------------------------------------------------------
# bias in the epilogue
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("ydt", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("variant", [-1, 10, 2])
def test_linear_bias(bits, ydt, variant):
    """fq_linear_bias: y = acc * s_x * s_w + bias[n].  Tolerance: the product and the sum are each rounded
    to fp32 (2^-24 of |product| and of |y|), then the output type's half ulp of |y|; measured against
    |product| + |bias| so that cancellation between the two does not inflate the ratio."""
    L = _layer("cfg3", M_override=300, K_override=1024, N_override=264)
    M, K = L.X.shape
    N = L.W.shape[0]
    align = 128 if bits == 8 else 256
    src, rep, kp, kpad = fq.fq_flatten_plan(L.chmax, L.T, align)
    Wq_ref, s_w_ref = O.flatten_weights(L.W, src, bits)
    acc_ref, _, s_x_ref = O.linear(L.X, src, rep, Wq_ref, s_w_ref, bits, want_y=False)
    rng = np.random.default_rng(3)
    prod = O.dequant(acc_ref, s_x_ref, s_w_ref)
    bias = (rng.standard_normal(N) * np.sqrt(np.mean(prod ** 2))).astype(np.float32)
    y_ref = O.dequant_bias(acc_ref, s_x_ref, s_w_ref, bias)
    lay = fq.FqLinear(to_dev(L.W_store, L.spec.w_dtype), L.chmax, L.T, bits, device=DEV)
    tdt = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[ydt]
    Y = torch.full((M, N), 7.0, dtype=tdt, device=DEV)
    ws = bytes_ws(fq.fq_linear_workspace_bytes(M, K, lay.Kpad, bits))
    fq.fq_gemm_select(variant)
    try:
        fq.fq_linear_bias(to_dev(L.X_store, L.spec.x_dtype), lay.src, lay.rep, lay.Wq, lay.s_w,
                          torch.from_numpy(bias).to(DEV), bits, Y, ws)
        torch.cuda.synchronize()
    finally:
        fq.fq_gemm_select(-1)
    got = Y.float().cpu().numpy().astype(np.float64)
    tol = {"f32": 1e-6, "f16": 1e-3, "bf16": 2.0 ** -8}[ydt]
    denom = np.abs(prod) + np.abs(bias.astype(np.float64))[None, :] + 1e-300
    assert (np.abs(got - y_ref) / denom).max() <= tol
    # a NULL bias is the plain call
    Y0 = torch.empty((M, N), dtype=torch.float32, device=DEV)
    Y1 = torch.empty((M, N), dtype=torch.float32, device=DEV)
    X = to_dev(L.X_store, L.spec.x_dtype)
    fq.fq_linear_bias(X, lay.src, lay.rep, lay.Wq, lay.s_w, None, bits, Y0, ws)
    fq.fq_linear(X, lay.src, lay.rep, lay.Wq, lay.s_w, bits, Y1, ws)
    torch.cuda.synchronize()
    assert torch.equal(Y0, Y1)


# ------------------------------------------------------------------------------------------
# maps that do not come from the plan functions (the kernel's general paths)
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("static", [False, True])
def test_flatten_quant_act_irregular_map(bits, static):
    """Any (src_idx, rep) is a valid map: head groups that are not the identity, appended slots whose
    copy count differs from their channel's, sources beyond the last full group of 16, padding in the
    middle.  The fast paths must not be taken for these, and the result still equals the definition."""
    rng = np.random.default_rng(42 + bits)
    M, K, Kpad = 77, 200, 512                                  # K % 16 = 8: channels 192..199 have no full head group
    X = (rng.standard_normal((M, K)) * rng.choice([1, 1, 10], K)).astype(np.float32)
    src = np.full(Kpad, -1, dtype=np.int32)
    rep = np.zeros(Kpad, dtype=np.int32)
    src[:K] = np.arange(K)
    rep[:K] = rng.integers(1, 4, K)
    src[16:32] = src[16:32][::-1]                               # a head group that is a permutation
    src[40] = 7                                                 # a head slot pointing elsewhere
    rep[40] = rep[7]
    tail = np.arange(K + 8, 420)
    src[tail] = rng.integers(0, K, tail.size)
    rep[tail] = rep[src[tail]]
    odd = tail[::5]
    rep[odd] = rep[src[odd]] + 1                                # copy count differs from the channel's own slot
    src[300:316] = -1                                           # a padding group in the middle
    rep[300:316] = 0
    src[330:346] = 199                                          # a source outside the full head groups
    rep[330:346] = rep[199]
    a_ref = np.float32(3.0) if static else O.act_absmax_dynamic(X, src, rep)
    q_ref, s_ref = O.flatten_quant_act(X, src, rep, bits, a_ref)
    want = q_ref.view(np.uint8) if bits == 8 else O.pack_i4(q_ref)
    out = torch.full((M, Kpad if bits == 8 else Kpad // 2), 0x55, dtype=torch.uint8, device=DEV)
    s_x = torch.zeros(1, dtype=torch.float32, device=DEV)
    ws = bytes_ws(fq.fq_act_workspace_bytes(K, Kpad))
    fq.fq_flatten_quant_act(torch.from_numpy(X).to(DEV), dev_i32(src), dev_i32(rep), bits, out, s_x, ws,
                            absmax_in=scalar(3.0) if static else None)
    torch.cuda.synchronize()
    assert np.float32(s_x.item()) == s_ref
    np.testing.assert_array_equal(out.cpu().numpy(), want)


# ------------------------------------------------------------------------------------------
# the calls are capturable: no allocation, no synchronization, clears done by fill kernels
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("bits", [8, 4, 6])
def test_linear_replayed_from_a_graph(bits):
    """fq_linear captured once into a HIP graph and replayed with new inputs between replays: every
    replay equals the eager call on the same input (raw accumulators, so the comparison is exact).
    bits = 6: the 4-bit layer in E3M2 storage."""
    L = _layer("cfg3", M_override=300, K_override=1024, N_override=264)
    M, K = L.X.shape
    N = L.W.shape[0]
    lay = fq.FqLinear(to_dev(L.W_store, L.spec.w_dtype), L.chmax, L.T, bits, device=DEV)
    ws = bytes_ws(fq.fq_linear_workspace_bytes(M, K, lay.Kpad, bits))
    X = to_dev(L.X_store, L.spec.x_dtype).clone()
    Yg = torch.zeros((M, N), dtype=torch.int32, device=DEV)
    Ye = torch.zeros((M, N), dtype=torch.int32, device=DEV)
    fq.fq_linear(X, lay.src, lay.rep, lay.Wq, lay.s_w, bits, Yg, ws)      # first use outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        fq.fq_linear(X, lay.src, lay.rep, lay.Wq, lay.s_w, bits, Yg, ws)
    ws_e = bytes_ws(fq.fq_linear_workspace_bytes(M, K, lay.Kpad, bits))
    rng = np.random.default_rng(5)
    for rnd in range(4):
        scale = float(rng.uniform(0.3, 1.5))
        X.copy_((to_dev(L.X_store, L.spec.x_dtype).float() * scale).to(X.dtype))   # new contents, same buffer
        Yg.fill_(-1)
        graph.replay()
        torch.cuda.synchronize()
        fq.fq_linear(X, lay.src, lay.rep, lay.Wq, lay.s_w, bits, Ye, ws_e)
        torch.cuda.synchronize()
        assert torch.equal(Yg, Ye), f"replay {rnd} differs from the eager call"
    # and the eager result is the oracle's on the last input
    Xh = X.float().cpu().numpy()
    qbits = 4 if bits == 6 else bits
    Wq_ref, s_w_ref = O.flatten_weights(L.W, lay.src_host, qbits)
    acc_ref, _, _ = O.linear(Xh, lay.src_host, lay.rep_host, Wq_ref, s_w_ref, qbits, want_y=False)
    np.testing.assert_array_equal(Ye.cpu().numpy(), acc_ref)


@pytest.mark.parametrize("bits", [8, 4])
def test_gemm_more_tiles_than_compute_units(bits):
    """272 tiles of 256 x 256 with ragged edges: on a 256-CU device the large-problem kernel walks a
    second round (prefetching across the tile boundary) and finishes with half-height tiles."""
    rng = np.random.default_rng(900 + bits)
    M, N, Kpad = 17 * 256 - 20, 16 * 256 - 7, 160 if bits == 8 else 320
    Xq, Wq = _rand_q(rng, M, Kpad, bits), _rand_q(rng, N, Kpad, bits)
    ref = O.gemm_i32(Xq, Wq)
    assert np.array_equal(_gemm_acc(Xq, Wq, bits), ref)
    # the 2-byte staged epilogue of the same walk
    Xd = torch.from_numpy(Xq if bits == 8 else O.pack_i4(Xq)).to(DEV)
    Wd = torch.from_numpy(Wq if bits == 8 else O.pack_i4(Wq)).to(DEV)
    Npad = N + 7                                               # rows of Y on 16-byte boundaries
    Y = torch.zeros((M, Npad), dtype=torch.bfloat16, device=DEV)
    s_x, s_w = scalar(0.01), scalar(0.003)
    (fq.fq_gemm_i8 if bits == 8 else fq.fq_gemm_i4)(Xd, Wd, s_x, s_w, Y[:, :N])
    torch.cuda.synchronize()
    y_ref = O.dequant(ref, np.float32(0.01), np.float32(0.003))
    assert rel_err(bf16_to_f64(Y[:, :N]), y_ref).max() <= 2.0 ** -8
    assert not Y[:, N:].any()


# ------------------------------------------------------------------------------------------
# the four-wave kernel with 128 x 128 wave tiles (INT8 and bf16 only)
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("variant", [11, 12])
def test_gemm_four_wave_kernel_int8(variant):
    """Variants 11 and 12 (two stage buffers / A three deep and B two deep, copies staggered over the waves): raw accumulators on ragged shapes (masked last k-stage, one-stage and two-stage reductions),
    a grid with half-height tail tiles, the staged 2-byte epilogue with bias, and a batched launch."""
    rng = np.random.default_rng(1100)
    fq.fq_gemm_select(variant)
    try:
        for (M, N, Kpad) in [(300, 520, 384), (257, 129, 1152), (1, 1, 128), (33, 700, 256), (512, 256, 128), (70, 41, 640),
                             (17 * 256 - 20, 16 * 256 - 7, 256), (24 * 256 - 20, 22 * 256 - 7, 384)]:
            Xq, Wq = _rand_q(rng, M, Kpad, 8), _rand_q(rng, N, Kpad, 8)
            assert np.array_equal(_gemm_acc(Xq, Wq, 8), O.gemm_i32(Xq, Wq)), (M, N, Kpad)
        lo = -128
        Xq = np.full((40, 26112), lo, np.int8)
        Wq = np.full((70, 26112), lo, np.int8)
        Wq[1::2] = 127
        assert np.array_equal(_gemm_acc(Xq, Wq, 8), O.gemm_i32(Xq, Wq))
        # epilogue: bf16 with bias, padded row stride
        M, N, Kpad = 300, 333, 512
        Xq, Wq = _rand_q(rng, M, Kpad, 8), _rand_q(rng, N, Kpad, 8)
        s_x, s_w = np.float32(0.0123), np.float32(0.00071)
        bias = rng.normal(0, 3.0, N).astype(np.float32)
        Ybuf = torch.full((M, 384), 7.0, dtype=torch.bfloat16, device=DEV)
        fq.fq_gemm_i8_bias(torch.from_numpy(Xq).to(DEV), torch.from_numpy(Wq).to(DEV), scalar(s_x), scalar(s_w),
                           torch.from_numpy(bias).to(DEV), Ybuf[:, :N])
        torch.cuda.synchronize()
        acc = O.gemm_i32(Xq, Wq)
        prod = O.dequant(acc, s_x, s_w)
        denom = np.abs(prod) + np.abs(bias.astype(np.float64))[None, :] + 1e-300
        got = Ybuf[:, :N].float().cpu().numpy().astype(np.float64)
        assert (np.abs(got - O.dequant_bias(acc, s_x, s_w, bias)) / denom).max() <= 2.0 ** -8
        assert (Ybuf[:, N:].float() == 7.0).all()
        # batched
        Aq, Bq = _bmm_operands(7, 3, 260, 300, 256, 8)
        Y = torch.full((3, 260, 300), -1, dtype=torch.int32, device=DEV)
        fq.fq_bmm_i8(_to_dev_q(Aq, 8), _to_dev_q(Bq, 8), None, None, Y)
        torch.cuda.synchronize()
        assert np.array_equal(Y.cpu().numpy(), O.bmm_i32(Aq, Bq))
    finally:
        fq.fq_gemm_select(-1)


def test_gemm_four_wave_kernel_nibbles():
    """Variant 12 on packed nibbles (low pass / high pass per k-slice, widening interleaved with the MFMAs): raw
    accumulators on ragged shapes with one, two, three and more k-stages, the extreme codes at the longest row that the
    accumulator bound allows, a grid with half-height tail tiles, the bf16 epilogue with bias, a batched launch."""
    rng = np.random.default_rng(1300)
    fq.fq_gemm_select(12)
    try:
        for (M, N, Kpad) in [(300, 520, 768), (257, 129, 2304), (1, 1, 256), (33, 700, 512), (512, 256, 1280), (70, 41, 3328),
                             (17 * 256 - 20, 16 * 256 - 7, 512), (24 * 256 - 20, 22 * 256 - 7, 768)]:
            Xq, Wq = _rand_q(rng, M, Kpad, 4), _rand_q(rng, N, Kpad, 4)
            assert np.array_equal(_gemm_acc(Xq, Wq, 4), O.gemm_i32(Xq, Wq)), (M, N, Kpad)
        Xq = np.full((40, 65536), -8, np.int8)
        Wq = np.full((70, 65536), -8, np.int8)
        Wq[1::2] = 7
        Xq[:, 1::2] = 7                                             # low and high nibbles differ in every byte
        assert np.array_equal(_gemm_acc(Xq, Wq, 4), O.gemm_i32(Xq, Wq))
        M, N, Kpad = 300, 333, 1024
        Xq, Wq = _rand_q(rng, M, Kpad, 4), _rand_q(rng, N, Kpad, 4)
        s_x, s_w = np.float32(0.0123), np.float32(0.00071)
        bias = rng.normal(0, 3.0, N).astype(np.float32)
        Ybuf = torch.full((M, 384), 7.0, dtype=torch.bfloat16, device=DEV)
        fq.fq_gemm_i4_bias(torch.from_numpy(O.pack_i4(Xq)).to(DEV), torch.from_numpy(O.pack_i4(Wq)).to(DEV), scalar(s_x),
                           scalar(s_w), torch.from_numpy(bias).to(DEV), Ybuf[:, :N])
        torch.cuda.synchronize()
        want = O.dequant_out(O.gemm_i32(Xq, Wq), s_x, s_w, "bf16", bias)
        assert np.array_equal(bits16(Ybuf[:, :N]), want)
        assert (Ybuf[:, N:].float() == 7.0).all()
        Aq, Bq = _bmm_operands(9, 3, 260, 300, 512, 4)
        Y = torch.full((3, 260, 300), -1, dtype=torch.int32, device=DEV)
        fq.fq_bmm_i4(_to_dev_q(Aq, 4), _to_dev_q(Bq, 4), None, None, Y)
        torch.cuda.synchronize()
        assert np.array_equal(Y.cpu().numpy(), O.bmm_i32(Aq, Bq))
    finally:
        fq.fq_gemm_select(-1)


@pytest.mark.parametrize("bits,Kpad", [(8, 128), (8, 256), (8, 640), (4, 256), (4, 512), (4, 1280)])
def test_gemm_four_wave_kernel_several_rounds_bf16(bits, Kpad):
    """More than two rounds of whole tiles per CU plus half-height tail tiles, bf16 output, reductions of one, two
    and five stages (packed nibbles: a stage is 256 values).  Every stored bf16 against the oracle's bits."""
    rng = np.random.default_rng(1400 + bits + Kpad)
    M, N = 27 * 256, 21 * 256 + 128                         # 27 x 22 = 594 tiles: 512 whole + 82 -> 164 halves
    Xq, Wq = _rand_q(rng, M, Kpad, bits), _rand_q(rng, N, Kpad, bits)
    s_x, s_w = np.float32(0.0123), np.float32(0.00071)
    Y = torch.zeros((M, N), dtype=torch.bfloat16, device=DEV)
    fq.fq_gemm_select(12)
    try:
        (fq.fq_gemm_i8 if bits == 8 else fq.fq_gemm_i4)(_to_dev_2d(Xq, bits), _to_dev_2d(Wq, bits), scalar(s_x), scalar(s_w), Y)
        torch.cuda.synchronize()
    finally:
        fq.fq_gemm_select(-1)
    want = O.dequant_out(O.gemm_i32(Xq, Wq), s_x, s_w, "bf16")
    assert np.array_equal(bits16(Y), want)


@pytest.mark.parametrize("bits", [8, 4])
def test_gemm_four_wave_kernel_random_shapes(bits):
    """Variant 12 on 24 seeded random shapes (1..700 rows and columns, 1..12 k-stages, every tile raggedness): raw
    accumulators against the oracle, and the bf16 bits of the same product through the bf16-only instantiation."""
    rng = np.random.default_rng(1500 + bits)
    stage = 128 if bits == 8 else 256
    fq.fq_gemm_select(12)
    try:
        for case in range(24):
            M, N = int(rng.integers(1, 700)), int(rng.integers(1, 700))
            Kpad = stage * int(rng.integers(1, 13))
            Xq, Wq = _rand_q(rng, M, Kpad, bits), _rand_q(rng, N, Kpad, bits)
            ref = O.gemm_i32(Xq, Wq)
            assert np.array_equal(_gemm_acc(Xq, Wq, bits), ref), (case, M, N, Kpad)
            Npad = (N + 7) // 8 * 8
            Y = torch.full((M, Npad), 5.0, dtype=torch.bfloat16, device=DEV)
            s_x, s_w = np.float32(rng.uniform(1e-3, 1e-1)), np.float32(rng.uniform(1e-4, 1e-2))
            (fq.fq_gemm_i8 if bits == 8 else fq.fq_gemm_i4)(_to_dev_2d(Xq, bits), _to_dev_2d(Wq, bits), scalar(s_x), scalar(s_w), Y[:, :N])
            torch.cuda.synchronize()
            assert np.array_equal(bits16(Y[:, :N]), O.dequant_out(ref, s_x, s_w, "bf16")), (case, M, N, Kpad)
            assert (Y[:, N:].float() == 5.0).all()
    finally:
        fq.fq_gemm_select(-1)


def _to_dev_2d(q, bits):
    return torch.from_numpy(q if bits == 8 else O.pack_i4(q)).to(DEV)


def test_gemm_four_wave_kernels_reject_what_they_cannot_run():
    Y = torch.zeros((4, 4), dtype=torch.int32, device=DEV)
    try:
        fq.fq_gemm_select(11)
        Xq = torch.zeros((4, 128), dtype=torch.uint8, device=DEV)
        with pytest.raises(fq.FqError, match="FQ_ERR_RANGE"):              # no packed-nibble form of variant 11
            fq.fq_gemm_i4(Xq, Xq, None, None, Y)
        for variant in (11, 12):
            fq.fq_gemm_select(variant)
            X8 = torch.zeros((4, 160), dtype=torch.int8, device=DEV)      # 160-byte rows: a partial second stage
            with pytest.raises(fq.FqError, match="FQ_ERR_SHAPE"):
                fq.fq_gemm_i8(X8, X8, None, None, Y)
        X4 = torch.zeros((4, 80), dtype=torch.uint8, device=DEV)          # 160 nibbles: less than one stage
        with pytest.raises(fq.FqError, match="FQ_ERR_SHAPE"):
            fq.fq_gemm_i4(X4, X4, None, None, Y)
    finally:
        fq.fq_gemm_select(-1)


def test_gemm_int8_large_default_bf16_output():
    """272 tiles with whole-stage rows and a plain bf16 output: the automatic choice takes the four-wave kernel in
    its bf16-only instantiation (with half-height tail tiles); every output against the oracle."""
    rng = np.random.default_rng(1200)
    M, N, Kpad = 17 * 256 - 20, 16 * 256 - 7, 256
    Xq, Wq = _rand_q(rng, M, Kpad, 8), _rand_q(rng, N, Kpad, 8)
    Y = torch.zeros((M, N + 7), dtype=torch.bfloat16, device=DEV)
    fq.fq_gemm_i8(torch.from_numpy(Xq).to(DEV), torch.from_numpy(Wq).to(DEV), scalar(0.01), scalar(0.003), Y[:, :N])
    torch.cuda.synchronize()
    y_ref = O.dequant(O.gemm_i32(Xq, Wq), np.float32(0.01), np.float32(0.003))
    assert rel_err(bf16_to_f64(Y[:, :N]), y_ref).max() <= 2.0 ** -8
    assert not Y[:, N:].any()


# ------------------------------------------------------------------------------------------
# the kernels the benchmark times: large problems, plain bf16 output -> the instantiations that carry the
# bf16 epilogue only.  Their stored bits against the oracle's rounded output, element by element.
# ------------------------------------------------------------------------------------------
def _q_operands(rng, M, N, Kpad, storage):
    qbits = 8 if storage == 8 else 4
    Xq, Wq = _rand_q(rng, M, Kpad, qbits), _rand_q(rng, N, Kpad, qbits)
    if storage == 8:
        return Xq, Wq, torch.from_numpy(Xq).to(DEV), torch.from_numpy(Wq).to(DEV)
    if storage == 4:
        return Xq, Wq, torch.from_numpy(O.pack_i4(Xq)).to(DEV), torch.from_numpy(O.pack_i4(Wq)).to(DEV)
    return Xq, Wq, torch.from_numpy(O.pack_e3m2_blocked(Xq)).to(DEV), torch.from_numpy(O.pack_e3m2_blocked(Wq)).to(DEV)


@pytest.mark.parametrize("storage,Kpad", [(8, 512), (8, 416), (4, 1024), (4, 512), (6, 384)])
def test_large_problem_kernels_store_the_oracles_bf16_bits(storage, Kpad):
    """272 ragged tiles of 256 x 256 (a second round with half-height tail tiles on a 256-CU device), bf16 output,
    no bias, automatic kernel choice: INT8 with whole 128-byte stages -> the four-wave kernel, with a partial last
    stage -> the ping-pong kernel; nibbles with long / short rows -> long / short phases; E3M2 -> the four-wave
    6-bit kernel; each in its bf16-only instantiation."""
    rng = np.random.default_rng(7000 + 10 * storage + Kpad)
    M, N = 17 * 256 - 20, 16 * 256 - 7
    Xq, Wq, Xd, Wd = _q_operands(rng, M, N, Kpad, storage)
    s_x, s_w = np.float32(0.0123), np.float32(0.00071)
    Y = torch.zeros((M, N + 7), dtype=torch.bfloat16, device=DEV)      # rows of Y on 16-byte boundaries
    if storage == 8:
        fq.fq_gemm_i8(Xd, Wd, scalar(s_x), scalar(s_w), Y[:, :N])
    elif storage == 4:
        fq.fq_gemm_i4(Xd, Wd, scalar(s_x), scalar(s_w), Y[:, :N])
    else:
        fq.fq_gemm_i4_e3m2(Xd, Wd, scalar(s_x), scalar(s_w), None, Y[:, :N])
    torch.cuda.synchronize()
    acc = O.gemm_i32(Xq, Wq)
    assert np.array_equal(bits16(Y[:, :N]), O.dequant_out(acc, s_x, s_w, "bf16"))
    assert not Y[:, N:].any()


@pytest.mark.parametrize("storage,Kpad", [(8, 384), (4, 768), (6, 256)])
def test_exactly_representable_outputs_through_the_bf16_only_kernels(storage, Kpad):
    """Scales of 1 and sparse operands in {-1, 0, 1}: every accumulator has magnitude <= 256 and is a bf16 value
    itself, so the stored output must equal the integer accumulator exactly -- a wrong or dropped k-slice in any
    tile shows as a wrong integer."""
    rng = np.random.default_rng(7100 + storage)
    M, N = 17 * 256 - 20, 16 * 256 - 7
    Xq = (rng.integers(-1, 2, (M, Kpad)) * (rng.random((M, Kpad)) < 0.5)).astype(np.int8)
    Wq = (rng.integers(-1, 2, (N, Kpad)) * (rng.random((N, Kpad)) < 0.5)).astype(np.int8)
    if storage == 8:
        Xd, Wd = torch.from_numpy(Xq).to(DEV), torch.from_numpy(Wq).to(DEV)
    elif storage == 4:
        Xd, Wd = torch.from_numpy(O.pack_i4(Xq)).to(DEV), torch.from_numpy(O.pack_i4(Wq)).to(DEV)
    else:
        Xd, Wd = torch.from_numpy(O.pack_e3m2_blocked(Xq)).to(DEV), torch.from_numpy(O.pack_e3m2_blocked(Wq)).to(DEV)
    one = scalar(1.0)
    Y = torch.zeros((M, N + 7), dtype=torch.bfloat16, device=DEV)
    call = {8: lambda: fq.fq_gemm_i8(Xd, Wd, one, one, Y[:, :N]), 4: lambda: fq.fq_gemm_i4(Xd, Wd, one, one, Y[:, :N]),
            6: lambda: fq.fq_gemm_i4_e3m2(Xd, Wd, one, one, None, Y[:, :N])}[storage]
    call()
    torch.cuda.synchronize()
    acc = O.gemm_i32(Xq, Wq)
    assert np.abs(acc).max() <= 256
    assert np.array_equal(Y[:, :N].float().cpu().numpy(), acc.astype(np.float32))


@pytest.mark.parametrize("storage", [8, 4, 6])
@pytest.mark.parametrize("ydt", ["bf16", "f16", "f32"])
def test_biased_and_half_epilogues_store_the_oracles_bits(storage, ydt):
    """Large-problem kernels in their generic instantiation: bias, half and fp32 outputs, bit for bit."""
    rng = np.random.default_rng(7200 + storage)
    M, N, Kpad = 17 * 256 - 20, 16 * 256 - 8, 512
    Xq, Wq, Xd, Wd = _q_operands(rng, M, N, Kpad, storage)
    s_x, s_w = np.float32(0.0123), np.float32(0.00071)
    bias = rng.normal(0, 3.0, N).astype(np.float32)
    tdt = {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32}[ydt]
    Y = torch.zeros((M, N), dtype=tdt, device=DEV)
    bd = torch.from_numpy(bias).to(DEV)
    if storage == 8:
        fq.fq_gemm_i8_bias(Xd, Wd, scalar(s_x), scalar(s_w), bd, Y)
    elif storage == 4:
        fq.fq_gemm_i4_bias(Xd, Wd, scalar(s_x), scalar(s_w), bd, Y)
    else:
        fq.fq_gemm_i4_e3m2(Xd, Wd, scalar(s_x), scalar(s_w), bd, Y)
    torch.cuda.synchronize()
    exact = O.dequant_out(O.gemm_i32(Xq, Wq), s_x, s_w, ydt, bias=bias)
    if ydt == "f32":
        assert np.array_equal(bits32(Y), exact.view(np.uint32))
    else:
        assert np.array_equal(bits16(Y), exact)
