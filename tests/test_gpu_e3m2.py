"""GPU parity of the 4-bit layer in E3M2 storage (6-bit codes on the 6-bit matrix pipe): the quantizer's
bytes against the oracle's packer, the GEMM's accumulators against the oracle's integer GEMM."""
import numpy as np
import pytest
import torch

import fq_workloads as WL
import paper_2402_17985_amd as fq
from oracle import fq_oracle as O
from tests.gpu_util import DEV, bf16_to_f64, bytes_ws, dev_i32, rel_err, scalar, to_dev

pytestmark = pytest.mark.gpu
E3 = fq.binding.FQ_BITS_I4_E3M2


def _layer(cfg, idx=0, **over):
    return WL.make_layer(WL.CONFIGS[cfg], idx, **over)


VARIANTS = [-1]          # the 6-bit GEMM has one kernel (four waves, 128 x 128 wave tiles); the variant hook does not apply


def _acc(Xq, Wq, variant=-1):
    """int8 arrays of 4-bit values -> raw accumulators of the E3M2 GEMM."""
    M, N = Xq.shape[0], Wq.shape[0]
    Y = torch.full((M, N), -12345, dtype=torch.int32, device=DEV)
    fq.fq_gemm_select(variant)
    try:
        fq.fq_gemm_i4_e3m2(torch.from_numpy(O.pack_e3m2_blocked(Xq)).to(DEV),
                           torch.from_numpy(O.pack_e3m2_blocked(Wq)).to(DEV), None, None, None, Y)
        torch.cuda.synchronize()
    finally:
        fq.fq_gemm_select(-1)
    return Y.cpu().numpy()


def _rand_q4(rng, rows, Kpad):
    return rng.integers(-8, 8, (rows, Kpad), dtype=np.int8)


@pytest.mark.parametrize("static", [False, True])
@pytest.mark.parametrize("cfg,over", [
    ("cfg1", {}), ("cfg1b", {}),
    ("cfg2", dict(M_override=333, K_override=1000, N_override=8)),        # ragged M, K not a multiple of 16
    ("cfg3", dict(M_override=517, K_override=2048, N_override=8)),
    ("cfg4", dict(M_override=70, K_override=5120, N_override=8)),
])
def test_flatten_quant_act_e3m2_bytes(cfg, over, static):
    L = _layer(cfg, **over)
    if L.spec.x_dtype != "f32" and L.X.shape[1] % 8:
        pytest.skip("row stride must be a multiple of 16 bytes")
    src, rep, kp, kpad = O.plan(L.chmax, L.T, 128)
    M, K = L.X.shape
    a = np.float32(L.T) if static else O.act_absmax_dynamic(L.X, src, rep)
    q, s_x_o = O.flatten_quant_act(L.X, src, rep, 4, a)
    want = O.pack_e3m2_blocked(q)
    out = torch.full((kpad // 128, M, 96), 0x55, dtype=torch.uint8, device=DEV)
    s_x = torch.zeros(1, dtype=torch.float32, device=DEV)
    ws = bytes_ws(fq.fq_act_workspace_bytes(K, kpad))
    fq.fq_flatten_quant_act(to_dev(L.X_store, L.spec.x_dtype), dev_i32(src), dev_i32(rep), E3, out, s_x, ws,
                            absmax_in=scalar(a) if static else None)
    torch.cuda.synchronize()
    assert np.float32(s_x.item()) == s_x_o
    assert np.array_equal(out.cpu().numpy(), want)


def test_flatten_weights_e3m2_bytes():
    L = _layer("cfg2", M_override=64, K_override=1024, N_override=301)
    src, rep, kp, kpad = O.plan(L.chmax, L.T, 128)
    N, K = L.W.shape
    Wq_o, s_w_o = O.flatten_weights(L.W, src, 4)
    out = torch.full((kpad // 128, N, 96), 0x55, dtype=torch.uint8, device=DEV)
    s_w = torch.zeros(1, dtype=torch.float32, device=DEV)
    fq.fq_flatten_weights(to_dev(L.W_store, L.spec.w_dtype), dev_i32(src), E3, out, s_w,
                          bytes_ws(fq.fq_weights_workspace_bytes(K, kpad)))
    torch.cuda.synchronize()
    assert np.float32(s_w.item()) == s_w_o
    assert np.array_equal(out.cpu().numpy(), O.pack_e3m2_blocked(Wq_o))


@pytest.mark.parametrize("variant", VARIANTS)
def test_gemm_e3m2_accumulators_bit_exact(variant):
    rng = np.random.default_rng(61)
    # several tiles + ragged tails in M and N (also M, N not multiples of 4: blocks off the 128-byte grid);
    # Kpad = 128 is a single stage, 256 two stages (fewer than the ring holds), 384 exactly the ring
    for (M, N, Kpad) in [(300, 520, 512), (257, 129, 1152), (1, 1, 128), (33, 700, 256), (256, 256, 384), (70, 41, 640),
                         (513, 260, 4096)]:
        Xq, Wq = _rand_q4(rng, M, Kpad), _rand_q4(rng, N, Kpad)
        assert np.array_equal(_acc(Xq, Wq, variant), O.gemm_i32(Xq, Wq)), (variant, M, N, Kpad)


@pytest.mark.parametrize("variant", VARIANTS)
def test_gemm_e3m2_every_code_pair(variant):
    """All 16 x 16 products of 4-bit values, each in every one of the 64 k-positions of an MFMA slice."""
    vals = np.arange(-8, 8, dtype=np.int8)
    Kpad = 128
    Xq = np.zeros((16 * 64, Kpad), np.int8)
    for v in range(16):
        for p in range(64):
            Xq[v * 64 + p, 64 * (v & 1) + p] = vals[v]
    Wq = np.repeat(vals[:, None], Kpad, axis=1)
    got = _acc(Xq, Wq, variant)
    assert np.array_equal(got, O.gemm_i32(Xq, Wq))
    assert got[0 * 64 + 5, 0] == 64 and got[15 * 64 + 63, 0] == -56


@pytest.mark.parametrize("variant", VARIANTS)
def test_gemm_e3m2_extreme_values_stay_exact(variant):
    Kpad = 26112                                     # |acc| up to 64 * Kpad = 1.67e6 < 2^24
    Xq = np.full((40, Kpad), -8, np.int8)
    Wq = np.full((70, Kpad), -8, np.int8)
    Wq[1::2] = 7
    got = _acc(Xq, Wq, variant)
    assert np.array_equal(got, O.gemm_i32(Xq, Wq))
    assert got[0, 0] == 64 * Kpad and got[0, 1] == -56 * Kpad


def test_gemm_e3m2_widest_layer_stays_exact():
    """The largest accumulator magnitude the interface admits: Kpad just under 131072, every product 64."""
    Kpad = 131072 - 128
    Xq = np.full((3, Kpad), -8, np.int8)
    Wq = np.full((5, Kpad), -8, np.int8)
    Wq[1, ::3] = 7
    Wq[2, 5::7] = -3
    got = _acc(Xq, Wq)
    assert np.array_equal(got, O.gemm_i32(Xq, Wq))
    assert got[0, 0] == 64 * Kpad


@pytest.mark.parametrize("ydt,tol", [(torch.float32, 1e-6), (torch.float16, 1e-3), (torch.bfloat16, 2.0 ** -8)])
@pytest.mark.parametrize("with_bias", [False, True])
@pytest.mark.parametrize("variant", VARIANTS)
def test_gemm_e3m2_epilogue(ydt, tol, with_bias, variant):
    rng = np.random.default_rng(7)
    M, N, Kpad = 300, 333, 512
    Xq, Wq = _rand_q4(rng, M, Kpad), _rand_q4(rng, N, Kpad)
    s_x, s_w = np.float32(0.0123), np.float32(0.071)
    bias = rng.normal(0, 3.0, N).astype(np.float32)
    ldy = 384
    Ybuf = torch.full((M, ldy), 7.0, dtype=ydt, device=DEV)
    fq.fq_gemm_select(variant)
    try:
        fq.fq_gemm_i4_e3m2(torch.from_numpy(O.pack_e3m2_blocked(Xq)).to(DEV),
                           torch.from_numpy(O.pack_e3m2_blocked(Wq)).to(DEV), scalar(s_x), scalar(s_w),
                           torch.from_numpy(bias).to(DEV) if with_bias else None, Ybuf[:, :N])
        torch.cuda.synchronize()
    finally:
        fq.fq_gemm_select(-1)
    acc = O.gemm_i32(Xq, Wq)
    prod = O.dequant(acc, s_x, s_w)
    got = Ybuf[:, :N].float().cpu().numpy().astype(np.float64)
    if with_bias:
        # product and sum each rounded to fp32, then to the output type: measured against |product| + |bias|
        # so that cancellation between the two does not inflate the ratio
        ref = O.dequant_bias(acc, s_x, s_w, bias)
        denom = np.abs(prod) + np.abs(bias.astype(np.float64))[None, :] + 1e-300
        assert (np.abs(got - ref) / denom).max() <= tol
    else:
        assert rel_err(got, prod).max() <= tol
    assert (Ybuf[:, N:].float() == 7.0).all()


@pytest.mark.parametrize("cfg,over", [
    ("cfg1b", {}),
    ("cfg3", dict(M_override=384, K_override=1024, N_override=700)),
    ("cfg4", dict(M_override=260, K_override=2048, N_override=264)),
])
def test_linear_e3m2_end_to_end(cfg, over):
    """The whole layer in E3M2 storage gives the accumulators of the 4-bit oracle layer."""
    L = _layer(cfg, **over)
    src, rep, kp, kpad = O.plan(L.chmax, L.T, 128)
    Wq_o, s_w_o = O.flatten_weights(L.W, src, 4)
    acc_o, y_o, s_x_o = O.linear(L.X, src, rep, Wq_o, s_w_o, 4)
    lay = fq.FqLinear(to_dev(L.W_store, L.spec.w_dtype), L.chmax, L.T, E3)
    assert (lay.src_host == src).all() and (lay.rep_host == rep).all()
    Xd = to_dev(L.X_store, L.spec.x_dtype)
    acc = lay.forward(Xd, out_dtype=torch.int32)
    y16 = lay.forward(Xd, out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    assert np.array_equal(acc.cpu().numpy(), acc_o)
    assert rel_err(bf16_to_f64(y16), y_o).max() <= 2.0 ** -8
    acc_s, _, _ = O.linear(L.X, src, rep, Wq_o, s_w_o, 4, a_static=L.T)
    acc_sg = lay.forward(Xd, out_dtype=torch.int32, absmax_in=scalar(L.T))
    torch.cuda.synchronize()
    assert np.array_equal(acc_sg.cpu().numpy(), acc_s)


@pytest.mark.parametrize("variant", VARIANTS)
def test_gemm_e3m2_more_tiles_than_compute_units(variant):
    """A grid of several waves of workgroups: sampled rows and columns against the oracle."""
    rng = np.random.default_rng(11)
    M, N, Kpad = 4096 + 40, 4096 + 8, 640
    Xq, Wq = _rand_q4(rng, M, Kpad), _rand_q4(rng, N, Kpad)
    got = _acc(Xq, Wq, variant)
    rows = np.unique(np.concatenate([rng.integers(0, M, 48), [0, M - 1, 4095, 4096]]))
    cols = np.unique(np.concatenate([rng.integers(0, N, 48), [0, N - 1, 4095, 4096]]))
    assert np.array_equal(got[rows], O.gemm_i32(Xq[rows], Wq))
    assert np.array_equal(got[:, cols], O.gemm_i32(Xq, Wq[cols]))


def test_peel_split_has_no_e3m2_form():
    L = _layer("cfg1b")
    src, rep, kp, kpad = O.plan(L.chmax, L.T, 128)
    M, K = L.X.shape
    out = torch.zeros((kpad // 128, M, 96), dtype=torch.uint8, device=DEV)
    with pytest.raises(fq.FqError, match="FQ_ERR_DTYPE"):
        fq.fq_flatten_quant_act_peel(to_dev(L.X_store, L.spec.x_dtype), dev_i32(src), dev_i32(rep), E3, float(L.T), out,
                                     torch.zeros(1, dtype=torch.float32, device=DEV),
                                     bytes_ws(fq.fq_act_workspace_bytes(K, kpad)))
    torch.cuda.synchronize()


@pytest.mark.parametrize("Kpad", [128, 256, 384, 1024])
def test_gemm_e3m2_several_rounds_of_tiles(Kpad):
    """600 tiles on a 256-CU device: two rounds of full tiles and a round of half-height tiles; reductions of
    one, two, three (= the ring) and eight stages.  Sampled rows and columns against the oracle, bf16 epilogue."""
    rng = np.random.default_rng(1300 + Kpad)
    M, N = 25 * 256 - 20, 24 * 256 - 7
    Xq, Wq = _rand_q4(rng, M, Kpad), _rand_q4(rng, N, Kpad)
    got = _acc(Xq, Wq)
    rows = np.unique(np.concatenate([rng.integers(0, M, 40), [0, M - 1, 255, 256, 3071, 3072]]))
    cols = np.unique(np.concatenate([rng.integers(0, N, 40), [0, N - 1, 255, 256]]))
    assert np.array_equal(got[rows], O.gemm_i32(Xq[rows], Wq))
    assert np.array_equal(got[:, cols], O.gemm_i32(Xq, Wq[cols]))
    Y = torch.zeros((M, N + 7), dtype=torch.bfloat16, device=DEV)
    fq.fq_gemm_i4_e3m2(torch.from_numpy(O.pack_e3m2_blocked(Xq)).to(DEV), torch.from_numpy(O.pack_e3m2_blocked(Wq)).to(DEV),
                       scalar(0.01), scalar(0.003), None, Y[:, :N])
    torch.cuda.synchronize()
    y_ref = O.dequant(O.gemm_i32(Xq[rows], Wq), np.float32(0.01), np.float32(0.003))
    assert rel_err(bf16_to_f64(Y[torch.from_numpy(rows).to(DEV)][:, :N]), y_ref).max() <= 2.0 ** -8
    assert not Y[:, N:].any()


def test_two_sided_flatten_e3m2():
    """Weight-side flattening with both tensors in E3M2 storage: bytes, scales and accumulators bit-exact."""
    L = _layer("cfg3", M_override=300, K_override=1024, N_override=200)
    M, K = L.X.shape
    N = L.W.shape[0]
    rng = np.random.default_rng(9)
    W = L.W.copy()
    W[:, rng.choice(K, 12, replace=False)] *= np.float32(5.0)
    W_store, W = WL.round_to_dtype(W, L.spec.w_dtype)
    cw = np.abs(W).max(axis=0)
    T_w = float(np.float32(2.0 * np.median(cw)))
    src, rx, rw, od, kp, kpad = fq.fq_flatten_plan_xw(L.chmax, float(L.T), cw, T_w, align=128)
    assert (rw > 1).any() and (rx > 1).any()
    Wq_ref, s_w_ref = O.flatten_weights_split(W, src, rw, 4)
    Xq_ref, s_x_ref = O.flatten_quant_act(L.X, src, rx, 4, O.act_absmax_dynamic(L.X, src, rx))
    Wq = torch.full((kpad // 128, N, 96), 0x55, dtype=torch.uint8, device=DEV)
    Xq = torch.full((kpad // 128, M, 96), 0x55, dtype=torch.uint8, device=DEV)
    s_w, s_x = scalar(0.0), scalar(0.0)
    ws = bytes_ws(fq.fq_act_workspace_bytes(K, kpad))
    srcd = dev_i32(src)
    fq.fq_flatten_weights_split(to_dev(W_store, L.spec.w_dtype), srcd, dev_i32(rw), E3, Wq, s_w, ws)
    fq.fq_flatten_quant_act(to_dev(L.X_store, L.spec.x_dtype), srcd, dev_i32(rx), E3, Xq, s_x, ws)
    acc = torch.empty((M, N), dtype=torch.int32, device=DEV)
    fq.fq_gemm_i4_e3m2(Xq, Wq, None, None, None, acc)
    torch.cuda.synchronize()
    assert np.float32(s_w.item()) == s_w_ref and np.float32(s_x.item()) == s_x_ref
    np.testing.assert_array_equal(Wq.cpu().numpy(), O.pack_e3m2_blocked(Wq_ref))
    np.testing.assert_array_equal(Xq.cpu().numpy(), O.pack_e3m2_blocked(Xq_ref))
    np.testing.assert_array_equal(acc.cpu().numpy(), O.gemm_i32(Xq_ref, Wq_ref))


@pytest.mark.parametrize("variant", VARIANTS)
def test_gemm_e3m2_units_on_top_of_the_largest_sums(variant):
    """Exactness where it is tightest: accumulators close to the largest magnitude the interface admits (2^23),
    built from products of 64, with products of +-1, +-3 and +-7 mixed in, so that the result depends on the
    lowest bit of an fp32 accumulator that large.  Positions of the small products cover every k-slot of an
    MFMA and both ends of the reduction."""
    Kpad = 131072 - 128
    rng = np.random.default_rng(23)
    Xq = np.full((6, Kpad), -8, np.int8)
    Wq = np.full((9, Kpad), -8, np.int8)
    small = np.concatenate([np.arange(0, 64), rng.choice(np.arange(64, Kpad - 64), 501, replace=False),
                            np.arange(Kpad - 64, Kpad)])
    Xq[:, small] = rng.choice(np.array([1, -1], np.int8), (6, small.size))
    Wq[:, small] = rng.choice(np.array([1, -1, 3, -3, 7, -7], np.int8), (9, small.size))
    Wq[4] = -Wq[4]                                   # the same magnitudes on the negative side
    ref = O.gemm_i32(Xq, Wq)
    assert np.abs(ref).max() > (1 << 23) - (1 << 17) and (ref & 1).any()
    assert np.array_equal(_acc(Xq, Wq, variant), ref)
