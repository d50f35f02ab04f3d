"""Pins for the oracle's quantizer, INT4 storage and flatten arithmetic
(arXiv 2402.17985 Eq. 1; Sec. 4.1 Eq. 3-4)."""
import json
import os

import numpy as np
import pytest

from oracle import fq_oracle as O


@pytest.fixture(scope="module")
def cases(golden_dir):
    with open(os.path.join(golden_dir, "quant_cases.json")) as f:
        return json.load(f)


def _identity_map(K, align=32):
    src, rep, kp, kpad = O.plan(np.zeros(K, np.float32), 1.0, align)
    assert kp == K
    return src, rep


def test_dynamic_worked_example(cases):
    c = cases["dynamic_worked_example"]
    X = np.array(c["X"], np.float32)
    chmax = np.abs(X).max(axis=0)
    src, rep, kp, kpad = O.plan(chmax, c["T"], 32)
    a = O.act_absmax_dynamic(X, src, rep)
    assert float(a) == c["a_prime"]
    q, s_x = O.flatten_quant_act(X, src, rep, c["bits"], a)
    assert q[:, :kp].tolist() == c["Xq_head"]
    assert (q[:, kp:] == 0).all()
    assert s_x == np.float32(c["s_x_num"] / c["s_x_den"])


def test_static_ties_and_clamp_int8(cases):
    c = cases["static_ties_int8"]
    x = np.array([c["x"]], np.float32)
    src, rep = _identity_map(x.shape[1], 1)
    q, s_x = O.flatten_quant_act(x, src, rep, c["bits"], c["a_prime"])
    assert q[0].tolist() == c["q"]
    assert s_x == np.float32(1.0)


def test_static_int4_and_pack(cases):
    c = cases["static_int4"]
    x = np.array([c["x"]], np.float32)
    src, rep = _identity_map(x.shape[1], 2)
    q, _ = O.flatten_quant_act(x, src, rep, c["bits"], c["a_prime"])
    assert q[0].tolist() == c["q"]
    packed = O.pack_i4(q)
    assert [f"{b:02x}" for b in packed[0]] == c["packed_hex"]


def test_pack_hand_bytes_and_roundtrip(cases):
    c = cases["pack_bytes"]
    q = np.array(c["pairs"], np.int8)
    packed = O.pack_i4(q)
    assert [f"{b:02x}" for b in packed[:, 0]] == c["bytes_hex"]
    # all 256 byte values survive unpack -> pack, and unpack yields two's-complement nibbles
    allb = np.arange(256, dtype=np.uint8).reshape(256, 1)
    u = O.unpack_i4(allb)
    assert (O.pack_i4(u) == allb).all()
    for b in range(256):
        lo, hi = b & 15, b >> 4
        assert u[b, 0] == (lo - 16 if lo >= 8 else lo)
        assert u[b, 1] == (hi - 16 if hi >= 8 else hi)
    with pytest.raises(O.OracleError):
        O.pack_i4(np.array([[8, 0]], np.int8))


@pytest.mark.parametrize("bits", [8, 4])
def test_endpoints_and_dynamic_range(bits):
    """+-a' map to +-qmax exactly; the dynamic scale never produces qmin (Eq. 1 is symmetric)."""
    qmax = 2 ** (bits - 1) - 1
    rng = np.random.default_rng(bits)
    X = rng.standard_normal((37, 50)).astype(np.float32)
    X[:, 7] *= 40
    chmax = np.abs(X).max(axis=0)
    src, rep, kp, kpad = O.plan(chmax, 2.5, 32)
    a = O.act_absmax_dynamic(X, src, rep)
    q, s_x = O.flatten_quant_act(X, src, rep, bits, a)
    assert q.max() <= qmax and q.min() >= -qmax
    assert np.abs(q).max() == qmax            # the element that defines a' reaches the endpoint
    assert s_x == np.float32(np.float64(a) / qmax)
    # a' equals the maximum of the float64 flattened tensor rounded to fp32 per slot
    xf = O.flatten_float(X, src, rep)
    assert abs(float(a) - np.abs(xf).max()) <= 1e-6 * float(a)


@pytest.mark.parametrize("bits", [8, 4])
def test_integers_are_fixed_points(bits):
    """Integer data with a' = qmax (s = 1) quantizes to itself."""
    qmax = 2 ** (bits - 1) - 1
    vals = np.arange(-qmax, qmax + 1, dtype=np.float32).reshape(1, -1)
    if vals.shape[1] % 2:
        vals = np.concatenate([vals, [[0]]], axis=1).astype(np.float32)
    src, rep = _identity_map(vals.shape[1], 2)
    q, s_x = O.flatten_quant_act(vals, src, rep, bits, float(qmax))
    assert (q[0] == vals[0].astype(np.int8)).all()
    assert s_x == np.float32(1.0)


@pytest.mark.parametrize("bits", [8, 4])
def test_matches_textbook_per_tensor_quantizer_when_nothing_is_flattened(bits):
    """With T >= max|X| the method reduces to plain per-tensor quantization (Eq. 1), here
    evaluated in float64 as round(x / s).  The fp32 one-multiply form may differ from it only on
    the rare element whose scaled value lies within fp32 rounding of a tie, and then by 1."""
    qmax = 2 ** (bits - 1) - 1
    rng = np.random.default_rng(100 + bits)
    X = (rng.standard_normal((64, 96)) * 3).astype(np.float32)
    chmax = np.abs(X).max(axis=0)
    src, rep, kp, kpad = O.plan(chmax, float(chmax.max()), 32)
    assert kp == 96
    a = O.act_absmax_dynamic(X, src, rep)
    assert float(a) == float(chmax.max())
    q, s_x = O.flatten_quant_act(X, src, rep, bits, a)
    s = np.float64(chmax.max()) / qmax
    ideal = np.clip(np.rint(X.astype(np.float64) / s), -qmax - 1, qmax).astype(np.int64)
    diff = np.abs(q[:, :96].astype(np.int64) - ideal)
    assert diff.max() <= 1
    assert (diff != 0).mean() <= 1e-3


def test_copies_hold_equal_shares():
    """Every copy of a flattened channel holds the same code, and n * (x/n) restores x (Eq. 3,
    equal-split form) so that the repeated weight reproduces the product (Eq. 4)."""
    rng = np.random.default_rng(5)
    X = rng.standard_normal((9, 12)).astype(np.float32)
    X[:, 4] *= 30
    X[:, 10] *= 11
    chmax = np.abs(X).max(axis=0)
    T = 3.0
    src, rep, kp, kpad = O.plan(chmax, T, 32)
    xf = O.flatten_float(X, src, rep)
    assert np.abs(xf).max() <= T                      # the flattened maximum is bounded by T
    for j in range(12):
        slots = np.nonzero(src == j)[0]
        assert len(slots) == rep[j]
        np.testing.assert_allclose(xf[:, slots].sum(axis=1), X[:, j].astype(np.float64), rtol=1e-15)
        assert (xf[:, slots] == xf[:, slots[:1]]).all()
    a = O.act_absmax_dynamic(X, src, rep)
    q, _ = O.flatten_quant_act(X, src, rep, 8, a)
    for j in (4, 10):
        slots = np.nonzero(src == j)[0]
        assert (q[:, slots] == q[:, slots[:1]]).all()


def test_peel_split_of_the_printed_equation():
    """Eq. 3 as printed: floor(|x|/T) slots hold T, the next holds the remainder.  Pieces sum to
    x and never exceed T.  Hand case: T = 2, x = -5 -> [-2 | -2, -1]; x = 3 -> [2 | 1, 0]."""
    X = np.array([[1, -5, 0.5], [-2, 3, 0.25]], np.float32)
    src, rep, kp, kpad = O.plan(np.abs(X).max(axis=0), 2.0, 32)
    xp = O.flatten_float_peel(X, src, 2.0)
    assert xp[0, :5].tolist() == [1.0, -2.0, 0.5, -2.0, -1.0]
    assert xp[1, :5].tolist() == [-2.0, 2.0, 0.25, 1.0, 0.0]
    assert (xp[:, 5:] == 0).all()


def test_weights_quantize_then_repeat():
    """Eq. 1 on W (per tensor), then Eq. 4: column j of Wq appears at every slot of channel j."""
    W = np.array([[0.5, -1.0, 0.25], [1.0, 0.125, -0.75]], np.float32)     # max|W| = 1 -> 1/s = 127
    src = np.array([0, 1, 2, 1, 1, -1, -1, -1], np.int32)
    Wq, s_w = O.flatten_weights(W, src, 8)
    # 0.5*127 = 63.5 -> 64 (tie to even); 0.25*127 = 31.75 -> 32; 0.125*127 = 15.875 -> 16;
    # -0.75*127 = -95.25 -> -95
    assert Wq.tolist() == [[64, -127, 32, -127, -127, 0, 0, 0], [127, 16, -95, 16, 16, 0, 0, 0]]
    assert s_w == np.float32(1.0 / 127.0)
    Wq4, s_w4 = O.flatten_weights(W, src, 4)
    # 1/s = 7: 3.5 -> 4 (tie to even), -7, 1.75 -> 2; 7, 0.875 -> 1, -5.25 -> -5
    assert Wq4.tolist() == [[4, -7, 2, -7, -7, 0, 0, 0], [7, 1, -5, 1, 1, 0, 0, 0]]
    assert s_w4 == np.float32(1.0 / 7.0)
    Wz, s_z = O.flatten_weights(np.zeros((2, 3), np.float32), src, 8)
    assert (Wz == 0).all() and s_z == np.float32(1.0)


def test_e3m2_storage_hand_codes_and_round_trip():
    """The 6-bit E3M2 storage of 4-bit values.  Hand codes from the format (sign | exponent, bias 3 |
    two mantissa bits): 1 = 2^0 -> e=3 m=0 -> 0b001100; 3 = 2 * 1.5 -> e=4 m=2 -> 0b010010;
    5 = 4 * 1.25 -> 0b010101; 7 = 4 * 1.75 -> 0b010111; -8 = -(2^3) -> 0b111000; 0 -> 0.
    Bit stream, little endian: slots (1, 3, 5, 7) -> 0x0C | 0x12 << 6 | 0x15 << 12 | 0x17 << 18."""
    q = np.zeros((1, 16), dtype=np.int8)
    q[0, :6] = [1, 3, 5, 7, -8, -1]
    got = O.pack_e3m2(q)
    word = 0x0C | (0x12 << 6) | (0x15 << 12) | (0x17 << 18) | (0x38 << 24) | (0x2C << 30)
    want = np.frombuffer(int(word).to_bytes(12, "little"), dtype=np.uint8)
    assert got.shape == (1, 12) and got[0].tolist() == want.tolist()
    # every representable value decodes, by the format's definition, to itself
    allq = np.tile(np.arange(-8, 8, dtype=np.int8), (3, 2))              # [3, 32]
    dec = O.unpack_e3m2(O.pack_e3m2(allq))
    np.testing.assert_array_equal(dec, allq.astype(np.float64))
    # slots are independent 6-bit fields: changing one slot changes only its bits
    a, b = allq.copy(), allq.copy()
    b[1, 5] = 7 if a[1, 5] != 7 else 6
    diff = np.flatnonzero(O.pack_e3m2(a)[1] != O.pack_e3m2(b)[1])
    assert set(diff.tolist()) <= {3, 4}                                  # bits 30..35 live in bytes 3 and 4
    with pytest.raises(O.OracleError):
        O.pack_e3m2(np.full((1, 16), 9, dtype=np.int8))


def test_e3m2_blocked_layout_hand_addresses():
    """The blocked E3M2 layout: the 96 bytes of (block t, row r) sit at (t * rows + r) * 96; a 48-byte group
    is X_a Y_a Y_b X_b (X: stream bytes 0..15 of a 32-code unit, Y: bytes 16..23), units in order (0, 1) for
    rows with bit 4 clear, (1, 0) for rows with bit 4 set.  Hand case, 18 rows x 256 slots, zero except:
    q[1, 0] = 1 (code 0x0C; block 0, group 0, unit 0, stream byte 0 -> X_0 at +0)       -> byte 1*96 = 96;
    q[2, 128] = -8 (code 0x38; block 1, group 0, unit 0, stream byte 0)                  -> byte (18+2)*96 = 1920;
    q[0, 255] = 3 (code 0x12; block 1, group 1, unit 1, code 31 = stream bits 186..191 = byte 23 = Y_1[7],
                   Y_1 at +24)                                       -> byte 18*96 + 48 + 31 = 1807, value 0x12 << 2;
    q[17, 0] = 1 (row bit 4 set: unit 0 is stored second, X_0 at +32)                    -> byte 17*96 + 32 = 1664;
    q[16, 32] = 1 (unit 1, stored first in this row, X_1 at +0)                          -> byte 16*96 = 1536;
    q[16, 31] = 5 (code 0x15; unit 0, code 31 -> Y_0[7], Y_0 at +24 in this row)         -> byte 1536 + 31 = 1567."""
    q = np.zeros((18, 256), dtype=np.int8)
    q[1, 0], q[2, 128], q[0, 255], q[17, 0], q[16, 32], q[16, 31] = 1, -8, 3, 1, 1, 5
    blk = O.pack_e3m2_blocked(q)
    assert blk.shape == (2, 18, 96)
    want = np.zeros(2 * 18 * 96, dtype=np.uint8)
    want[96], want[1920], want[1807], want[1664], want[1536], want[1567] = 0x0C, 0x38, 0x12 << 2, 0x0C, 0x0C, 0x15 << 2
    assert np.flatnonzero(blk.reshape(-1)).tolist() == np.flatnonzero(want).tolist()
    assert blk.reshape(-1).tolist() == want.tolist()
    # a permutation of the plain stream's bytes, the same for all rows of equal bit 4 and for all blocks
    rng = np.random.default_rng(5)
    q = rng.integers(-8, 8, (40, 640), dtype=np.int8)
    blk, stream = O.pack_e3m2_blocked(q), O.pack_e3m2(q)
    fwd = list(range(0, 24)) + list(range(40, 48)) + list(range(24, 40))       # X0 Y0 Y1 X1
    rev = list(range(24, 48)) + list(range(16, 24)) + list(range(0, 16))       # X1 Y1 Y0 X0
    for t in range(5):
        for r in range(40):
            piece = stream[r, 96 * t:96 * t + 96]
            perm = fwd if (r & 16) == 0 else rev
            want_piece = np.concatenate([piece[:48][perm], piece[48:][perm]])
            assert blk[t, r].tolist() == want_piece.tolist()
    with pytest.raises(ValueError):
        O.pack_e3m2_blocked(np.zeros((2, 192), dtype=np.int8))
