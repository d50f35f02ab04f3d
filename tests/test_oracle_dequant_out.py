"""Pins for the oracle's output-type dequantization (arXiv 2402.17985 Sec. 2.1 Eq. 1 inverted,
applied to the integer product of Sec. 5.1; the layer hands a 16-bit tensor to the next operator).

Three kinds of pin: bit patterns worked by hand (ties in the last kept bit, carries into the exponent,
fp32 rounding of large accumulators before the 16-bit rounding, subnormal and overflowing halves, the
separately rounded bias add); NumPy's and PyTorch's own conversions to half and bfloat16 on random
values (library routines, not this repository's bit code); and the unrounded float64 dequantization,
which every output must lie within half a unit in the last place of."""
import json
import os
import struct

import numpy as np
import pytest

from oracle import fq_oracle as O


def _f32(hexstr):
    return np.float32(struct.unpack("<f", struct.pack("<I", int(hexstr, 16)))[0])


def _scales(c):
    s_x = _f32(c["s_x_hex"]) if "s_x_hex" in c else np.float32(c["s_x"])
    s_w = _f32(c["s_w_hex"]) if "s_w_hex" in c else np.float32(c["s_w"])
    return s_x, s_w


@pytest.fixture(scope="module")
def cases(golden_dir):
    with open(os.path.join(golden_dir, "dequant_out_cases.json")) as f:
        return json.load(f)


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_hand_bit_patterns_16bit(cases, dtype):
    for c in cases[dtype]:
        s_x, s_w = _scales(c)
        got = O.dequant_out(np.array([[c["acc"]]], np.int32), s_x, s_w, dtype)
        assert f"{int(got[0, 0]):04x}" == c["hex"], c["why"]


def test_hand_values_f32(cases):
    for c in cases["f32"]:
        s_x, s_w = _scales(c)
        got = O.dequant_out(np.array([[c["acc"]]], np.int32), s_x, s_w, "f32")
        assert got.dtype == np.float32 and float(got[0, 0]) == c["value"], c["why"]


def test_hand_values_with_bias(cases):
    for c in cases["bias"]:
        s_x, s_w = _scales(c)
        bias = np.array([_f32(c["bias_hex"])], np.float32)
        got = O.dequant_out(np.array([[c["acc"]]], np.int32), s_x, s_w, c["dtype"], bias=bias)
        width = 8 if c["dtype"] == "f32" else 4
        assert f"{int(got.view(np.uint32 if width == 8 else np.uint16)[0, 0]):0{width}x}" == c["hex"], c["why"]


def test_against_library_conversions():
    """fp32 steps with NumPy's float32 scalars, half through NumPy's astype, bfloat16 through PyTorch's."""
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(11)
    acc = np.concatenate([rng.integers(-2**31, 2**31, 4000), rng.integers(-70000, 70000, 4000),
                          rng.integers(-300, 300, 2000)]).astype(np.int32).reshape(100, 100)
    bias = (rng.standard_normal(100) * 3).astype(np.float32)
    for s_x, s_w in ((np.float32(0.0123), np.float32(0.00071)), (np.float32(1.0), np.float32(1.0)),
                     (np.float32(3.1e-5), np.float32(2.9e-4))):
        scale = np.float32(s_x * s_w)
        for b in (None, bias):
            f = acc.astype(np.float32) * scale                 # NumPy: int32 -> float32 is round-to-nearest-even
            if b is not None:
                f = f + b[None, :]
            assert f.dtype == np.float32
            assert np.array_equal(O.dequant_out(acc, s_x, s_w, "f32", bias=b).view(np.uint32), f.view(np.uint32))
            with np.errstate(over="ignore"):
                h = f.astype(np.float16).view(np.uint16)
            assert np.array_equal(O.dequant_out(acc, s_x, s_w, "f16", bias=b), h)
            bf = torch.from_numpy(f).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
            assert np.array_equal(O.dequant_out(acc, s_x, s_w, "bf16", bias=b), bf)


def test_all_halves_are_fixed_points_and_midpoints_tie_to_even():
    """Every finite half value converts to itself; the midpoint of two neighbours goes to the even one."""
    pats = np.arange(0, 0x7c00, dtype=np.uint16)                       # all non-negative finite halves
    vals = pats.view(np.float16).astype(np.float32)
    one = np.float32(1.0)
    # feed fp32 values through the bias (acc = 0): f = fl32(0 + bias) = bias
    got = O.dequant_out(np.zeros((1, len(vals)), np.int32), one, one, "f16", bias=vals)
    assert np.array_equal(got[0], pats)
    mid = ((vals[:-1].astype(np.float64) + vals[1:].astype(np.float64)) / 2).astype(np.float32)   # exact in fp32
    got = O.dequant_out(np.zeros((1, len(mid)), np.int32), one, one, "f16", bias=mid)
    expect = np.where(pats[:-1] % 2 == 0, pats[:-1], pats[1:])
    assert np.array_equal(got[0], expect)


def test_within_half_ulp_of_the_float64_value():
    rng = np.random.default_rng(5)
    acc = rng.integers(-2**22, 2**22, (50, 60)).astype(np.int32)
    s_x, s_w = np.float32(0.031), np.float32(0.0042)
    y64 = O.dequant(acc, s_x, s_w)
    bf = O.dequant_out(acc, s_x, s_w, "bf16")
    ybf = (bf.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    assert (np.abs(ybf - y64) <= np.abs(y64) * (2.0 ** -8 + 2.0 ** -22)).all()
    h = O.dequant_out(acc, s_x, s_w, "f16").view(np.float16).astype(np.float64)
    assert (np.abs(h - y64) <= np.abs(y64) * (2.0 ** -11 + 2.0 ** -22) + 2.0 ** -25).all()
    f = O.dequant_out(acc, s_x, s_w, "f32").astype(np.float64)
    assert (np.abs(f - y64) <= np.abs(y64) * 2.0 ** -22).all()


def test_rejects_bad_arguments():
    import ctypes
    one = ctypes.c_float(1.0)
    acc = np.zeros((1, 1), np.int32)
    out = np.zeros((1, 1), np.float32)
    f = O.lib().fqo_dequant_out
    pa, po = acc.ctypes.data_as(ctypes.c_void_p), out.ctypes.data_as(ctypes.c_void_p)
    assert f(None, 1, 1, one, one, None, 2, po) != 0
    assert f(pa, 0, 1, one, one, None, 2, po) != 0
    assert f(pa, 1, 1, one, one, None, 3, po) != 0
    assert f(pa, 1, 1, one, one, None, 0, po) == 0
