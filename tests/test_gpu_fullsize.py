"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times
(FqLinear defaults: automatic kernel choice, 128/256-channel row alignment, dynamic scale).

What is compared: the flatten map, the quantized activations and weights and the scales in full
(bit-exact); the int32 accumulators on about 256 sampled rows and 256 sampled columns that the oracle
recomputes (bit-exact)
plus an exact int64 Freivalds identity over the whole matrix (acc r == Xq (Wq^T r) for a random
vector r: any wrong accumulator changes the left side unless its r entry is 0, probability 2^-20
per vector); the bf16 outputs on the sampled rows (relative 2^-8, see test_gpu_parity)."""
import numpy as np
import pytest
import torch

import fq_workloads as WL
import paper_2402_17985_amd as fq
from oracle import fq_oracle as O
from tests.gpu_util import DEV, bf16_to_f64, bits16, rel_err, to_dev

pytestmark = pytest.mark.gpu


E3 = fq.binding.FQ_BITS_I4_E3M2


def _check_layer(cfg_name, idx, n_sample_rows=256, n_sample_cols=256, freivalds=2, e3m2=False):
    """e3m2: the 4-bit layer in E3M2 storage on the 6-bit matrix pipe (what bench.py times for 4-bit layers):
    same quantized integers as the nibble path, other bytes, other GEMM kernel."""
    cfg = WL.CONFIGS[cfg_name]
    print(f"[fullsize] generating {cfg_name} layer {idx}", flush=True)
    L = WL.make_layer(cfg, idx)
    sp = L.spec
    bits = sp.bits
    print(f"[fullsize] {cfg_name}.{sp.name} M={sp.M} K={sp.K} N={sp.N} bits={bits}", flush=True)
    assert not e3m2 or bits == 4
    Wd = to_dev(L.W_store, sp.w_dtype)
    lay = fq.FqLinear(Wd, L.chmax, L.T, E3 if e3m2 else bits)
    Xd = to_dev(L.X_store, sp.x_dtype)
    stored = (lambda q: O.pack_e3m2_blocked(q).reshape(-1)) if e3m2 else \
             (lambda q: (q.view(np.uint8) if bits == 8 else O.pack_i4(q)).reshape(-1))
    # --- map, weights ---
    src, rep, kp, kpad = O.plan(L.chmax, L.T, 128 if (bits == 8 or e3m2) else 256)
    assert (lay.src_host == src).all() and (lay.rep_host == rep).all() and lay.Kpad == kpad
    Wq_o, s_w_o = O.flatten_weights(L.W, src, bits)
    Wq_g = lay.Wq.cpu().numpy().view(np.uint8).reshape(-1)
    assert np.float32(lay.s_w.item()) == s_w_o
    assert np.array_equal(Wq_g, stored(Wq_o))
    print("[fullsize]   map, weights and s_w equal the oracle's", flush=True)
    # --- quantized activations (the workspace of fq_linear starts with X'q) ---
    acc_g = lay.forward(Xd, out_dtype=torch.int32)
    torch.cuda.synchronize()
    cols = kpad // 4 * 3 if e3m2 else (kpad if bits == 8 else kpad // 2)
    Xq_g = lay.workspace(sp.M)[: sp.M * cols].cpu().numpy()
    a = O.act_absmax_dynamic(L.X, src, rep)
    Xq_o, s_x_o = O.flatten_quant_act(L.X, src, rep, bits, a)
    assert np.array_equal(Xq_g, stored(Xq_o))
    acc_g = acc_g.cpu().numpy()
    print("[fullsize]   quantized activations equal the oracle's", flush=True)
    # --- sampled rows, recomputed by the oracle ---
    rng = np.random.default_rng(12345 + idx)
    rows = np.unique(np.concatenate([[0, sp.M - 1, 255, 256], rng.integers(0, sp.M, n_sample_rows)]))
    acc_o = O.gemm_i32(Xq_o[rows], Wq_o)
    assert np.array_equal(acc_g[rows], acc_o)
    print(f"[fullsize]   {len(rows)} sampled accumulator rows equal the oracle's", flush=True)
    cols_s = np.unique(np.concatenate([[0, sp.N - 1], rng.integers(0, sp.N, n_sample_cols)]))
    assert np.array_equal(acc_g[:, cols_s], O.gemm_i32(Xq_o, Wq_o[cols_s]))
    print(f"[fullsize]   {len(cols_s)} sampled accumulator columns equal the oracle's", flush=True)
    # --- every accumulator at once: exact Freivalds identity in int64 ---
    for rep_i in range(freivalds):
        r = rng.integers(0, 1 << 20, sp.N).astype(np.int64)
        lhs = acc_g.astype(np.int64) @ r
        t = r @ Wq_o.astype(np.int64)
        rhs = Xq_o.astype(np.int64) @ t
        assert np.array_equal(lhs, rhs)
        print("[fullsize]   Freivalds identity holds over the whole accumulator matrix", flush=True)
    # --- dequantized bf16 output on the samples ---
    Y = lay.forward(Xd, out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    y_o = O.dequant(acc_o, s_x_o, s_w_o)
    Yrows = Y[torch.from_numpy(rows).to(DEV)]
    assert rel_err(bf16_to_f64(Yrows), y_o).max() <= 2.0 ** -8           # sanity against the unrounded value
    # the stored bf16 bits of the timed kernel (bf16 output, no bias) equal the oracle's rounded output
    assert np.array_equal(bits16(Yrows), O.dequant_out(acc_o, s_x_o, s_w_o, "bf16"))
    acc_cols = O.gemm_i32(Xq_o, Wq_o[cols_s])
    assert np.array_equal(bits16(Y[:, torch.from_numpy(cols_s).to(DEV)]), O.dequant_out(acc_cols, s_x_o, s_w_o, "bf16"))
    print("[fullsize]   bf16 output bits equal the oracle's on the sampled rows and columns", flush=True)


def test_cfg2_full():
    """LLaMA-7B q/k/v-style projection, INT8, M = 2048: every accumulator recomputed by the oracle."""
    L = WL.make_layer(WL.CONFIGS["cfg2"], 0)
    lay = fq.FqLinear(to_dev(L.W_store, "bf16"), L.chmax, L.T, 8)
    acc = lay.forward(to_dev(L.X_store, "bf16"), out_dtype=torch.int32)
    torch.cuda.synchronize()
    Wq_o, s_w_o = O.flatten_weights(L.W, lay.src_host, 8)
    acc_o, y_o, s_x_o = O.linear(L.X, lay.src_host, lay.rep_host, Wq_o, s_w_o, 8)
    assert np.array_equal(acc.cpu().numpy(), acc_o)
    Y = lay.forward(to_dev(L.X_store, "bf16"), out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    assert rel_err(bf16_to_f64(Y), y_o).max() <= 2.0 ** -8


@pytest.mark.parametrize("cfg,idx", [("cfg3", 0), ("cfg3", 1), ("cfg3i8", 0)])
def test_benchmark_layers_full_size(cfg, idx):
    _check_layer(cfg, idx)


@pytest.mark.parametrize("cfg,idx,e3m2", [("cfg2", 0, False), ("cfg3", 0, False), ("cfg3", 1, False), ("cfg3i8", 0, False),
                                          ("cfg3", 0, True), ("cfg3", 1, True)])
def test_timed_call_stores_the_oracles_bf16_bits_whole_matrix(cfg, idx, e3m2):
    """The call bench.py times (fq_linear, dynamic scale, bf16 output, automatic kernel choice) against the
    oracle's whole layer, every output element: the stored bf16 bit patterns are equal."""
    L = WL.make_layer(WL.CONFIGS[cfg], idx)
    sp = L.spec
    print(f"[fullsize] whole-matrix bf16 bits: {cfg}.{sp.name} M={sp.M} K={sp.K} N={sp.N} bits={sp.bits} e3m2={e3m2}", flush=True)
    lay = fq.FqLinear(to_dev(L.W_store, sp.w_dtype), L.chmax, L.T, E3 if e3m2 else sp.bits)
    Y = lay.forward(to_dev(L.X_store, sp.x_dtype))
    torch.cuda.synchronize()
    assert Y.dtype == torch.bfloat16
    got = bits16(Y)
    del Y
    src, rep, kp, kpad = O.plan(L.chmax, L.T, 128 if (sp.bits == 8 or e3m2) else 256)
    Wq_o, s_w_o = O.flatten_weights(L.W, src, sp.bits)
    acc_o, _, s_x_o = O.linear(L.X, src, rep, Wq_o, s_w_o, sp.bits, want_y=False)
    print("[fullsize]   oracle layer done", flush=True)
    assert np.array_equal(got, O.dequant_out(acc_o, s_x_o, s_w_o, "bf16"))


@pytest.mark.parametrize("cfg,idx", [("cfg3", 0), ("cfg3", 1), ("cfg4", 2), ("cfg5", 3), ("cfgP", 1)])
def test_four_bit_layers_in_e3m2_storage_full_size(cfg, idx):
    """The 4-bit layers as the benchmark runs them: E3M2 storage, 6-bit matrix pipe."""
    _check_layer(cfg, idx, freivalds=1, e3m2=True)


@pytest.mark.parametrize("idx", [0, 1, 2, 3])
def test_cfg4_opt13b_layers_full_size(idx):
    """OPT-13B-style layer, M = 8192: QKV and out projections INT8, FC1 / FC2 INT4."""
    _check_layer("cfg4", idx, freivalds=1)


@pytest.mark.parametrize("idx", [0, 1, 2, 3])
def test_cfg5_llama65b_layers_full_size(idx):
    """LLaMA-65B-scale layer, M = 16384: attention projections INT8, FFN INT4."""
    _check_layer("cfg5", idx, freivalds=1)


@pytest.mark.parametrize("idx", [0, 1])
def test_paper_table5_shape_full_size(idx):
    """The shape of the paper's operator measurement (Table 5): 8 x 2048 tokens, 4096 -> 4096, about 1024
    expanded channels; INT8 and INT4."""
    _check_layer("cfgP", idx, freivalds=1)
