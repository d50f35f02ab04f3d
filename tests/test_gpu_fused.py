"""fq_linear_fused_a_i8 (flatten + quantize fused into the GEMM's A-operand load; Sec. 6) against the oracle through
the C ABI: accumulators bit-exact, every output type's stored bits, static and dynamic scale, ragged shapes, a map
that does not come from the plan functions."""
import numpy as np
import pytest
import torch

import fq_workloads as WL
import paper_2402_17985_amd as fq
from oracle import fq_oracle as O
from tests.gpu_util import DEV, bits16, bits32, bytes_ws, dev_i32, scalar, to_dev

pytestmark = pytest.mark.gpu


def _run(Xd, src, rep, Wq, s_w, M, N, K, ydt, bias=None, a_static=None):
    Y = torch.full((M, N + 8), -3.0 if ydt != torch.int32 else -3, dtype=ydt, device=DEV)
    ws = bytes_ws(fq.fq_act_workspace_bytes(K, len(src)))
    fq.fq_linear_fused_a_i8(Xd, dev_i32(src), dev_i32(rep), torch.from_numpy(Wq).to(DEV), scalar(s_w), Y[:, :N], ws,
                            bias=None if bias is None else torch.from_numpy(bias).to(DEV),
                            absmax_in=None if a_static is None else scalar(a_static))
    torch.cuda.synchronize()
    assert (Y[:, N:] == -3).all()
    return Y[:, :N]


@pytest.mark.parametrize("shape", [(300, 1024, 264), (129, 200, 70), (1, 64, 1), (260, 4096, 515)])
@pytest.mark.parametrize("static", [False, True])
def test_fused_layer_equals_the_oracle(shape, static):
    M, K, N = shape
    L = WL.make_layer(WL.CONFIGS["cfg3i8"], 0, M_override=M, K_override=K, N_override=N)
    src, rep, kp, kpad = fq.fq_flatten_plan(L.chmax, L.T, 32)
    Wq, s_w = O.flatten_weights(L.W, src, 8)
    a_static = np.float32(L.T) if static else None
    acc_ref, _, s_x_ref = O.linear(L.X, src, rep, Wq, s_w, 8, a_static=a_static, want_y=False)
    Xd = to_dev(L.X_store, "bf16")
    got = _run(Xd, src, rep, Wq, s_w, M, N, K, torch.int32, a_static=a_static)
    assert np.array_equal(got.cpu().numpy(), acc_ref)
    rng = np.random.default_rng(M + N)
    bias = rng.normal(0, 2.0, N).astype(np.float32)
    for ydt, name in ((torch.bfloat16, "bf16"), (torch.float16, "f16"), (torch.float32, "f32")):
        for b in (None, bias):
            y = _run(Xd, src, rep, Wq, s_w, M, N, K, ydt, bias=b, a_static=a_static)
            want = O.dequant_out(acc_ref, s_x_ref, s_w, name, b)
            assert np.array_equal(bits32(y) if name == "f32" else bits16(y), want.view(np.uint32) if name == "f32" else want), (name, b is not None)


def test_fused_layer_with_a_map_not_from_the_plan():
    """Appended slots in arbitrary order, padding in the middle, a permuted head group: the gathered path."""
    rng = np.random.default_rng(77)
    M, K, N, Kpad = 77, 200, 40, 512
    X = (rng.standard_normal((M, K)) * rng.choice([1, 1, 10], K)).astype(np.float32)
    Xb = torch.from_numpy(X).to(DEV).to(torch.bfloat16)
    Xh = Xb.float().cpu().numpy()
    W = (rng.standard_normal((N, K)) * 0.05).astype(np.float32)
    src = np.full(Kpad, -1, dtype=np.int32)
    rep = np.zeros(Kpad, dtype=np.int32)
    src[:K] = np.arange(K)
    rep[:K] = rng.integers(1, 4, K)
    src[16:32] = src[16:32][::-1]
    tail = np.arange(K + 8, 420)
    src[tail] = rng.integers(0, K, tail.size)
    rep[tail] = rep[src[tail]]
    src[300:316] = -1
    rep[300:316] = 0
    Wq, s_w = O.flatten_weights(W, src, 8)
    acc_ref, _, s_x_ref = O.linear(Xh, src, rep, Wq, s_w, 8, want_y=False)
    got = _run(Xb, src, rep, Wq, s_w, M, N, K, torch.int32)
    assert np.array_equal(got.cpu().numpy(), acc_ref)
    y = _run(Xb, src, rep, Wq, s_w, M, N, K, torch.bfloat16)
    assert np.array_equal(bits16(y), O.dequant_out(acc_ref, s_x_ref, s_w, "bf16"))


def test_fused_layer_is_the_unfused_layer_bit_for_bit():
    L = WL.make_layer(WL.CONFIGS["cfg3i8"], 0, M_override=520, K_override=2048, N_override=384)
    lay = fq.FqLinear(to_dev(L.W_store, L.spec.w_dtype), L.chmax, L.T, 8, device=DEV)
    M, K = L.X.shape
    N = L.W.shape[0]
    X = to_dev(L.X_store, "bf16")
    Y0 = torch.empty((M, N), dtype=torch.bfloat16, device=DEV)
    Y1 = torch.empty((M, N), dtype=torch.bfloat16, device=DEV)
    fq.fq_linear(X, lay.src, lay.rep, lay.Wq, lay.s_w, 8, Y0, bytes_ws(fq.fq_linear_workspace_bytes(M, K, lay.Kpad, 8)))
    fq.fq_linear_fused_a_i8(X, lay.src, lay.rep, lay.Wq, lay.s_w, Y1, bytes_ws(fq.fq_act_workspace_bytes(K, lay.Kpad)))
    torch.cuda.synchronize()
    assert torch.equal(Y0.view(torch.int16), Y1.view(torch.int16))


def test_fused_layer_rejects_other_input_types():
    X = torch.zeros((4, 64), dtype=torch.float16, device=DEV)
    src = torch.arange(64, dtype=torch.int32, device=DEV)
    rep = torch.ones(64, dtype=torch.int32, device=DEV)
    Wq = torch.zeros((4, 64), dtype=torch.int8, device=DEV)
    Y = torch.zeros((4, 4), dtype=torch.float32, device=DEV)
    with pytest.raises(fq.FqError, match="FQ_ERR_DTYPE"):
        fq.fq_linear_fused_a_i8(X, src, rep, Wq, scalar(1.0), Y, bytes_ws(fq.fq_act_workspace_bytes(64, 64)))
