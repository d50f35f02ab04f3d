"""The C-ABI library loads, exports every entry point include/*.h declares, and its host-side
logic (argument validation, the flatten plan) behaves as documented.  No GPU needed."""
import ctypes
import json
import os
import re

import numpy as np
import pytest

import paper_2402_17985_amd as fq
from oracle import fq_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    names = set()
    for header in sorted(os.listdir(os.path.join(ROOT, "include"))):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(fq_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_every_declared_symbol_is_exported():
    L = fq.lib()
    names = _declared_symbols()
    assert len(names) >= 12
    for n in names:
        assert hasattr(L, n), n
    assert sorted(fq.SYMBOLS) == names
    assert fq.fq_version() >= 100


def test_plan_matches_oracle_on_hand_cases(golden_dir):
    cases = json.load(open(os.path.join(golden_dir, "plan_cases.json")))["cases"]
    for c in cases:
        src, rep, kp, kpad = fq.fq_flatten_plan(np.array(c["chmax"], np.float32), c["T"], c["align"])
        assert (kp, kpad) == (c["Kprime"], c["Kpad"])
        assert src[:kp].tolist() == c["src_head"] and rep[:kp].tolist() == c["rep_head"]
        assert (src[kp:] == -1).all() and (rep[kp:] == 0).all()


@pytest.mark.parametrize("seed", range(8))
def test_plan_matches_oracle_random(seed):
    rng = np.random.default_rng(seed)
    K = int(rng.integers(1, 3000))
    chmax = np.abs(rng.standard_normal(K)).astype(np.float32) * 4
    chmax[rng.integers(0, K, max(1, K // 50))] *= np.float32(rng.uniform(5, 200))
    if seed % 2:
        chmax[rng.integers(0, K, 3)] = 0.0
    T = float(np.float32(rng.uniform(0.5, 12.0)))
    if seed == 3:                       # exact multiples of T
        chmax[:5] = np.float32(T) * np.arange(1, 6, dtype=np.float32)
    align = int(rng.choice([32, 64, 128]))
    got = fq.fq_flatten_plan(chmax, T, align)
    want = O.plan(chmax, T, align)
    assert got[2:] == want[2:]
    assert (got[0] == want[0]).all() and (got[1] == want[1]).all()


def test_plan_argument_errors():
    L = fq.lib()
    good = np.ones(4, np.float32)
    kp, kpad = ctypes.c_int(), ctypes.c_int()
    call = lambda ch, K, T, al, cap=0: L.fq_flatten_plan(ch.ctypes.data if ch is not None else None, K, T, al,
                                                         None, None, cap, ctypes.byref(kp), ctypes.byref(kpad))
    assert call(None, 4, 1.0, 32) == 1                      # FQ_ERR_NULL
    assert call(good, 0, 1.0, 32) == 2                      # FQ_ERR_SHAPE
    assert call(good, 4, 1.0, 0) == 2
    for T in (0.0, -2.0, float("nan"), float("inf")):
        assert call(good, 4, T, 32) == 4                    # FQ_ERR_RANGE
    assert b"T" in L.fq_last_error_string()
    for bad in (np.array([1, np.nan, 1, 1], np.float32), np.array([1, -1, 1, 1], np.float32),
                np.array([np.inf, 1, 1, 1], np.float32)):
        assert call(bad, 4, 1.0, 32) == 4
    assert call(good, 4, 1.0, 32, cap=8) == 1               # cap > 0 with NULL outputs
    src = np.empty(8, np.int32)
    rep = np.empty(8, np.int32)
    rc = L.fq_flatten_plan(good.ctypes.data, 4, 1.0, 32, src.ctypes.data, rep.ctypes.data, 8, ctypes.byref(kp),
                           ctypes.byref(kpad))
    assert rc == 2 and kpad.value == 32                     # capacity too small, sizes still reported
    with pytest.raises(fq.FqError):
        fq.fq_flatten_plan(good, -1.0)


def test_device_calls_validate_before_launching():
    """Bad arguments are rejected on the host: these return before any HIP call is made."""
    L = fq.lib()
    dummy = 0x1000                                          # aligned, never dereferenced
    # NULL pointers
    assert L.fq_gemm_i8(None, dummy, 4, 4, 32, dummy, dummy, dummy, fq.FQ_F32, 4, None) == 1
    # Kpad not a multiple of 32
    assert L.fq_gemm_i8(dummy, dummy, 4, 4, 48, dummy, dummy, dummy, fq.FQ_F32, 4, None) == 2
    # accumulator overflow bound
    assert L.fq_gemm_i8(dummy, dummy, 4, 4, 131072, dummy, dummy, dummy, fq.FQ_F32, 4, None) == 4
    # bad output dtype, stride, alignment, missing scales
    assert L.fq_gemm_i4(dummy, dummy, 4, 4, 32, dummy, dummy, dummy, 9, 4, None) == 3
    assert L.fq_gemm_i4(dummy, dummy, 4, 4, 32, dummy, dummy, dummy, fq.FQ_F32, 3, None) == 2
    assert L.fq_gemm_i8(dummy + 4, dummy, 4, 4, 32, dummy, dummy, dummy, fq.FQ_F32, 4, None) == 5
    assert L.fq_gemm_i8(dummy, dummy, 4, 4, 32, None, dummy, dummy, fq.FQ_BF16, 4, None) == 1
    # activation path: dtype, bits, stride multiple of 16 bytes, workspace size
    ws = fq.fq_act_workspace_bytes(64, 64)
    assert ws > 0
    args = lambda dt=fq.FQ_BF16, ld=64, bits=8, wsb=ws: (dummy, dt, 4, 64, ld, dummy, dummy, 64, bits, None, dummy,
                                                        dummy, dummy, wsb, None)
    assert L.fq_flatten_quant_act(*args(dt=fq.FQ_I32)) == 3
    assert L.fq_flatten_quant_act(*args(bits=5)) == 3
    assert L.fq_flatten_quant_act(*args(ld=60)) == 2
    assert L.fq_flatten_quant_act(*args(ld=68)) == 2         # 136 bytes: not a multiple of 16
    assert L.fq_flatten_quant_act(*args(wsb=ws - 1)) == 7
    assert b"workspace" in L.fq_last_error_string()
    assert L.fq_gemm_bf16(dummy, dummy, 4, 4, 12, dummy, 4, None) == 2
    # batched product: batch count, operand strides (size, 16-byte multiple), output stride
    bmm = lambda batch=2, sa=128, sb=128, sy=16, f=L.fq_bmm_i8: f(dummy, dummy, batch, 4, 4, 32, sa, sb, dummy, dummy,
                                                                  dummy, fq.FQ_F32, 4, sy, None)
    assert bmm(batch=0) == 4
    assert bmm(batch=70000) == 4
    assert bmm(sa=64) == 2
    assert bmm(sb=136) == 5
    assert bmm(sy=15) == 2
    assert bmm(sa=32, f=L.fq_bmm_i4) == 2                    # a packed 4 x 32 matrix is 64 bytes
    assert L.fq_channel_absmax(dummy, fq.FQ_BF16, 4, 64, 60, 0, dummy, None) == 2
    assert L.fq_channel_absmax(dummy, fq.FQ_BF16, 4, 64, 64, 0, None, None) == 1
    assert L.fq_gemm_select(1700) == 4
    assert L.fq_gemm_select(0) == 4                          # a variant that no longer exists
    assert L.fq_gemm_select(-1) == 0
    assert fq.fq_linear_workspace_bytes(8, 64, 64, 8) >= 8 * 64 + ws
    assert fq.fq_linear_workspace_bytes(8, 64, 64, 4) >= 8 * 32 + ws
    # E3M2 storage of the 4-bit layer: Kpad a multiple of 128 (whole blocks), 3 bytes per 4 slots
    e3 = fq.binding.FQ_BITS_I4_E3M2
    assert L.fq_gemm_i4_e3m2(dummy, dummy, 4, 4, 96, dummy, dummy, None, dummy, fq.FQ_F32, 4, None) == 2
    assert b"multiple of 128" in L.fq_last_error_string()
    assert L.fq_gemm_i4_e3m2(dummy, None, 4, 4, 128, dummy, dummy, None, dummy, fq.FQ_F32, 4, None) == 1
    assert L.fq_gemm_i4_e3m2(dummy, dummy, 4, 4, 128, dummy, dummy, dummy, dummy, fq.FQ_I32, 4, None) == 3   # bias + raw
    args96 = (dummy, fq.FQ_BF16, 4, 64, 64, dummy, dummy, 96, e3, None, dummy, dummy, dummy, 1 << 20, None)
    assert L.fq_flatten_quant_act(*args96) == 2
    assert fq.fq_linear_workspace_bytes(8, 64, 128, e3) >= 8 * 96 + fq.fq_act_workspace_bytes(64, 128)


@pytest.mark.parametrize("seed", range(4))
def test_policy_helpers_match_oracle(seed):
    """Threshold (Eq. 6-7) and smoothing factors (Eq. 5): host functions of the library against the oracle."""
    rng = np.random.default_rng(seed)
    K = int(rng.integers(3, 2000))
    cx = (np.abs(rng.standard_normal(K)) * 4).astype(np.float32)
    cx[rng.integers(0, K, max(1, K // 100))] *= np.float32(rng.uniform(10, 100))
    cw = (np.abs(rng.standard_normal(K)) * 0.1 + 0.05).astype(np.float32)
    T = fq.fq_threshold_boxplot(cx, 1.3)
    assert abs(T - float(O.threshold_boxplot(cx, 1.3))) <= 1e-6 * T
    s = fq.fq_smooth_scales(cx, cw, 0.5)
    np.testing.assert_allclose(s, O.smooth_scales(cx, cw, 0.5), rtol=1e-6)
    # the hand cases of the oracle's pins
    assert fq.fq_threshold_boxplot(np.array([1, 2, 3, 4, 100], np.float32), 1.3) == float(np.float32(4.42))
    assert fq.fq_smooth_scales(np.array([5, 5], np.float32), np.array([1, 2], np.float32)).tolist() == [1.0, 1.0]
    with pytest.raises(fq.FqError):
        fq.fq_threshold_boxplot(cx, -1.0)
    with pytest.raises(fq.FqError):
        fq.fq_smooth_scales(cx, cw, 2.0)


@pytest.mark.parametrize("seed", range(6))
def test_plan_xw_matches_oracle(seed):
    """Two-sided plan (Sec. 4.1): the library's host function against the oracle, with and without weight maxima."""
    rng = np.random.default_rng(200 + seed)
    K = int(rng.integers(1, 600))
    cx = (np.abs(rng.standard_normal(K)) * rng.choice([1, 1, 1, 25], K)).astype(np.float32)
    cw = (np.abs(rng.standard_normal(K)) * 0.1 * rng.choice([1, 1, 4], K)).astype(np.float32)
    T_x, T_w = float(np.float32(rng.uniform(0.5, 4))), float(np.float32(rng.uniform(0.05, 0.3)))
    align = int(rng.choice([1, 32, 128, 256]))
    for w in (None, cw):
        got = fq.fq_flatten_plan_xw(cx, T_x, w, T_w, align)
        ref = O.plan_xw(cx, T_x, w, T_w, align)
        assert got[4:] == ref[4:]
        for a, b in zip(got[:4], ref[:4]):
            np.testing.assert_array_equal(a, b)
    with pytest.raises(fq.FqError):
        fq.fq_flatten_plan_xw(cx, 0.0)
    with pytest.raises(fq.FqError):
        fq.fq_flatten_plan_xw(cx, 1.0, cw, float("inf"))


def test_runtime_failures_come_back_as_fq_err_hip():
    """Error path of the device calls, forced from the host: on a machine without a GPU every HIP call fails, and the
    entry points must hand that back as FQ_ERR_HIP with the runtime's message (no crash, nothing thrown across the
    C boundary).  With a GPU present these calls would launch on dummy pointers, so the test runs only without one."""
    import torch
    if torch.cuda.is_available():
        pytest.skip("needs a machine without a GPU: the failing runtime is the forced condition")
    L = fq.lib()
    dummy = 0x10000
    ws = fq.fq_act_workspace_bytes(64, 64)
    calls = [
        lambda: L.fq_gemm_i8(dummy, dummy, 4, 4, 32, dummy, dummy, dummy, fq.FQ_F32, 4, None),
        lambda: L.fq_gemm_i4(dummy, dummy, 4, 4, 32, dummy, dummy, dummy, fq.FQ_BF16, 8, None),
        lambda: L.fq_flatten_quant_act(dummy, fq.FQ_BF16, 4, 64, 64, dummy, dummy, 64, 8, None, dummy, dummy, dummy, ws, None),
        lambda: L.fq_flatten_quant_act_noalloc(dummy, fq.FQ_BF16, 4, 64, 64, dummy, dummy, 64, 8, None, dummy, dummy, None),
        lambda: L.fq_channel_absmax(dummy, fq.FQ_BF16, 4, 64, 64, 0, dummy, None),
        lambda: L.fq_gemm_bf16(dummy, dummy, 4, 4, 16, dummy, 4, None),
    ]
    for call in calls:
        assert call() == 6                                   # FQ_ERR_HIP
        assert L.fq_last_error_string()                     # the runtime's own message is kept
    with pytest.raises(fq.FqError, match="FQ_ERR_HIP"):
        fq.binding._check(calls[0]())
