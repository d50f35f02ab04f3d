"""ctypes front end of the CPU oracle (oracle/fq_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
CPU-baseline leg.  It holds no arithmetic of the method: it marshals NumPy arrays into the C
functions, which are the definitions written from the paper (arXiv 2402.17985, Sec. 2.1 Eq. 1,
Sec. 4.1 Eq. 2-4, Sec. 5.1).  Nothing in the GPU package imports this module.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        _lib = ctypes.CDLL(path)
        _lib.fqo_absmax.restype = ctypes.c_float
        _lib.fqo_act_absmax_dynamic.restype = ctypes.c_float
        _lib.fqo_dot_i32.restype = ctypes.c_int32
        _lib.fqo_act_absmax_peel.restype = ctypes.c_float
    return _lib


def _p(a, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


class OracleError(RuntimeError):
    pass


def _check(rc, what):
    if rc != 0:
        raise OracleError(f"{what} failed with code {rc}")


def num_threads() -> int:
    return int(lib().fqo_num_threads())


def plan(chmax, T, align=32):
    """Eq. 2 / Eq. 3 index layout / padding.  Returns (src, rep, Kprime, Kpad)."""
    chmax = _f32(chmax)
    K = chmax.shape[0]
    kp, kpad = ctypes.c_int(0), ctypes.c_int(0)
    rc = lib().fqo_plan(_p(chmax, ctypes.c_float), K, ctypes.c_float(T), align, None, None, 0,
                        ctypes.byref(kp), ctypes.byref(kpad))
    _check(rc, "fqo_plan(size query)")
    src = np.empty(kpad.value, dtype=np.int32)
    rep = np.empty(kpad.value, dtype=np.int32)
    rc = lib().fqo_plan(_p(chmax, ctypes.c_float), K, ctypes.c_float(T), align,
                        _p(src, ctypes.c_int32), _p(rep, ctypes.c_int32), kpad.value,
                        ctypes.byref(kp), ctypes.byref(kpad))
    _check(rc, "fqo_plan")
    return src, rep, kp.value, kpad.value


def absmax(v) -> float:
    v = _f32(v).reshape(-1)
    return float(lib().fqo_absmax(_p(v, ctypes.c_float), ctypes.c_longlong(v.size)))


def flatten_weights(W, src, bits):
    """Eq. 1 + Eq. 4.  Returns (Wq int8 [N, Kpad], s_w)."""
    W = _f32(W)
    N, K = W.shape
    src = np.ascontiguousarray(src, dtype=np.int32)
    Kpad = src.shape[0]
    out = np.empty((N, Kpad), dtype=np.int8)
    s_w = ctypes.c_float(0)
    rc = lib().fqo_flatten_weights(_p(W, ctypes.c_float), N, K, _p(src, ctypes.c_int32), Kpad, bits,
                                   _p(out, ctypes.c_int8), ctypes.byref(s_w))
    _check(rc, "fqo_flatten_weights")
    return out, np.float32(s_w.value)


def act_absmax_dynamic(X, src, rep) -> np.float32:
    X = _f32(X)
    M, K = X.shape
    src = np.ascontiguousarray(src, dtype=np.int32)
    rep = np.ascontiguousarray(rep, dtype=np.int32)
    return np.float32(lib().fqo_act_absmax_dynamic(_p(X, ctypes.c_float), M, K, K,
                                                   _p(src, ctypes.c_int32), _p(rep, ctypes.c_int32),
                                                   src.shape[0]))


def flatten_quant_act(X, src, rep, bits, a_prime):
    """Eq. 3 (equal split) + Eq. 1.  Returns (Xq int8 [M, Kpad], s_x)."""
    X = _f32(X)
    M, K = X.shape
    src = np.ascontiguousarray(src, dtype=np.int32)
    rep = np.ascontiguousarray(rep, dtype=np.int32)
    Kpad = src.shape[0]
    out = np.empty((M, Kpad), dtype=np.int8)
    s_x = ctypes.c_float(0)
    rc = lib().fqo_flatten_quant_act(_p(X, ctypes.c_float), M, K, K, _p(src, ctypes.c_int32),
                                     _p(rep, ctypes.c_int32), Kpad, bits, ctypes.c_float(a_prime),
                                     _p(out, ctypes.c_int8), ctypes.byref(s_x))
    _check(rc, "fqo_flatten_quant_act")
    return out, np.float32(s_x.value)


def flatten_float(X, src, rep):
    X = _f32(X)
    M, K = X.shape
    src = np.ascontiguousarray(src, dtype=np.int32)
    rep = np.ascontiguousarray(rep, dtype=np.int32)
    out = np.empty((M, src.shape[0]), dtype=np.float64)
    lib().fqo_flatten_float(_p(X, ctypes.c_float), M, K, K, _p(src, ctypes.c_int32),
                            _p(rep, ctypes.c_int32), src.shape[0], _p(out, ctypes.c_double))
    return out


def flatten_float_peel(X, src, T):
    X = _f32(X)
    M, K = X.shape
    src = np.ascontiguousarray(src, dtype=np.int32)
    out = np.empty((M, src.shape[0]), dtype=np.float64)
    lib().fqo_flatten_float_peel(_p(X, ctypes.c_float), M, K, K, _p(src, ctypes.c_int32),
                                 src.shape[0], ctypes.c_double(T), _p(out, ctypes.c_double))
    return out


def repeat_weights_float(W, src):
    W = _f32(W)
    N, K = W.shape
    src = np.ascontiguousarray(src, dtype=np.int32)
    out = np.empty((N, src.shape[0]), dtype=np.float64)
    lib().fqo_repeat_weights_float(_p(W, ctypes.c_float), N, K, _p(src, ctypes.c_int32),
                                   src.shape[0], _p(out, ctypes.c_double))
    return out


def pack_i4(q):
    q = np.ascontiguousarray(q, dtype=np.int8)
    rows, Kpad = q.shape
    out = np.empty((rows, Kpad // 2), dtype=np.uint8)
    rc = lib().fqo_pack_i4(_p(q, ctypes.c_int8), ctypes.c_longlong(rows), Kpad, _p(out, ctypes.c_uint8))
    _check(rc, "fqo_pack_i4")
    return out


def unpack_i4(packed):
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    rows, half = packed.shape
    out = np.empty((rows, 2 * half), dtype=np.int8)
    rc = lib().fqo_unpack_i4(_p(packed, ctypes.c_uint8), ctypes.c_longlong(rows), 2 * half,
                             _p(out, ctypes.c_int8))
    _check(rc, "fqo_unpack_i4")
    return out


def gemm_i32(Xq, Wq, row0=0, rows=None):
    """acc[i, n] = sum_p Xq[i, p] * Wq[n, p] for rows [row0, row0+rows)."""
    Xq = np.ascontiguousarray(Xq, dtype=np.int8)
    Wq = np.ascontiguousarray(Wq, dtype=np.int8)
    M, Kpad = Xq.shape
    N, Kpad2 = Wq.shape
    assert Kpad == Kpad2
    if rows is None:
        rows = M - row0
    out = np.empty((rows, N), dtype=np.int32)
    rc = lib().fqo_gemm_i32(_p(Xq, ctypes.c_int8), _p(Wq, ctypes.c_int8), M, N, Kpad, row0, rows,
                            _p(out, ctypes.c_int32))
    _check(rc, "fqo_gemm_i32")
    return out


def dot_i32(x, w) -> int:
    x = np.ascontiguousarray(x, dtype=np.int8)
    w = np.ascontiguousarray(w, dtype=np.int8)
    assert x.shape == w.shape and x.ndim == 1
    return int(lib().fqo_dot_i32(_p(x, ctypes.c_int8), _p(w, ctypes.c_int8), x.shape[0]))


def dequant(acc, s_x, s_w):
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    out = np.empty(acc.shape, dtype=np.float64)
    lib().fqo_dequant(_p(acc, ctypes.c_int32), ctypes.c_longlong(acc.size), ctypes.c_float(s_x),
                      ctypes.c_float(s_w), _p(out, ctypes.c_double))
    return out


def linear_f64(X, W):
    X = _f32(X)
    W = _f32(W)
    M, K = X.shape
    N = W.shape[0]
    out = np.empty((M, N), dtype=np.float64)
    lib().fqo_linear_f64(_p(X, ctypes.c_float), _p(W, ctypes.c_float), M, N, K, K, _p(out, ctypes.c_double))
    return out


def matmul_nt_f64(A, B):
    A = np.ascontiguousarray(A, dtype=np.float64)
    B = np.ascontiguousarray(B, dtype=np.float64)
    M, Kp = A.shape
    N = B.shape[0]
    out = np.empty((M, N), dtype=np.float64)
    lib().fqo_matmul_nt_f64(_p(A, ctypes.c_double), _p(B, ctypes.c_double), M, N, Kp, _p(out, ctypes.c_double))
    return out


def linear(X, src, rep, Wq, s_w, bits, a_static=None, row0=0, rows=None, want_y=True):
    """The whole layer on rows [row0, row0+rows).  Returns (acc int32, y float64 or None, s_x)."""
    X = _f32(X)
    M, K = X.shape
    src = np.ascontiguousarray(src, dtype=np.int32)
    rep = np.ascontiguousarray(rep, dtype=np.int32)
    Wq = np.ascontiguousarray(Wq, dtype=np.int8)
    N, Kpad = Wq.shape
    assert Kpad == src.shape[0]
    if rows is None:
        rows = M - row0
    acc = np.empty((rows, N), dtype=np.int32)
    y = np.empty((rows, N), dtype=np.float64) if want_y else None
    s_x = ctypes.c_float(0)
    rc = lib().fqo_linear(_p(X, ctypes.c_float), M, K, K, _p(src, ctypes.c_int32), _p(rep, ctypes.c_int32),
                          Kpad, _p(Wq, ctypes.c_int8), ctypes.c_float(s_w), N, bits,
                          ctypes.c_float(-1.0 if a_static is None else a_static), row0, rows,
                          _p(acc, ctypes.c_int32), _p(y, ctypes.c_double) if want_y else None,
                          ctypes.byref(s_x))
    _check(rc, "fqo_linear")
    return acc, y, np.float32(s_x.value)


def threshold_boxplot(chmax, beta=1.3) -> np.float32:
    """Eq. 6-7: box-plot clipped mean of the channel maxima times beta."""
    chmax = _f32(chmax)
    T = ctypes.c_float(0)
    rc = lib().fqo_threshold_boxplot(_p(chmax, ctypes.c_float), chmax.shape[0], ctypes.c_float(beta), ctypes.byref(T))
    _check(rc, "fqo_threshold_boxplot")
    return np.float32(T.value)


def smooth_scales(chmax_x, chmax_w, alpha=0.5):
    """Eq. 5: per-channel smoothing factors s (X / s, s * W)."""
    chmax_x, chmax_w = _f32(chmax_x), _f32(chmax_w)
    assert chmax_x.shape == chmax_w.shape
    out = np.empty(chmax_x.shape[0], dtype=np.float32)
    rc = lib().fqo_smooth_scales(_p(chmax_x, ctypes.c_float), _p(chmax_w, ctypes.c_float), chmax_x.shape[0],
                                 ctypes.c_float(alpha), _p(out, ctypes.c_float))
    _check(rc, "fqo_smooth_scales")
    return out


def channel_absmax(X, prev=None):
    """Per-channel max |x| of X [M, K]; with prev [K] the running maximum max(prev, .)."""
    X = _f32(X)
    M, K = X.shape
    out = np.zeros(K, dtype=np.float32) if prev is None else _f32(prev).copy()
    rc = lib().fqo_channel_absmax(_p(X, ctypes.c_float), M, K, K, 0 if prev is None else 1, _p(out, ctypes.c_float))
    _check(rc, "fqo_channel_absmax")
    return out


def bmm_i32(Aq, Bq):
    """acc[b, i, n] = sum_p Aq[b, i, p] * Bq[b, n, p] (int8 operands, int32 result)."""
    Aq = np.ascontiguousarray(Aq, dtype=np.int8)
    Bq = np.ascontiguousarray(Bq, dtype=np.int8)
    batch, M, Kpad = Aq.shape
    batch2, N, Kpad2 = Bq.shape
    assert batch == batch2 and Kpad == Kpad2
    out = np.empty((batch, M, N), dtype=np.int32)
    rc = lib().fqo_bmm_i32(_p(Aq, ctypes.c_int8), _p(Bq, ctypes.c_int8), batch, M, N, Kpad, _p(out, ctypes.c_int32))
    _check(rc, "fqo_bmm_i32")
    return out


def plan_xw(chmax_x, T_x, chmax_w=None, T_w=1.0, align=32):
    """Two-sided plan.  Returns (src, rep_x, rep_w, ord, Kprime, Kpad)."""
    chmax_x = _f32(chmax_x)
    K = chmax_x.shape[0]
    cw = None if chmax_w is None else _f32(chmax_w)
    pw = None if cw is None else _p(cw, ctypes.c_float)
    kp, kpad = ctypes.c_int(0), ctypes.c_int(0)
    rc = lib().fqo_plan_xw(_p(chmax_x, ctypes.c_float), ctypes.c_float(T_x), pw, ctypes.c_float(T_w), K, align,
                           None, None, None, None, 0, ctypes.byref(kp), ctypes.byref(kpad))
    _check(rc, "fqo_plan_xw(size query)")
    arrs = [np.empty(kpad.value, dtype=np.int32) for _ in range(4)]
    rc = lib().fqo_plan_xw(_p(chmax_x, ctypes.c_float), ctypes.c_float(T_x), pw, ctypes.c_float(T_w), K, align,
                           *[_p(a, ctypes.c_int32) for a in arrs], kpad.value, ctypes.byref(kp), ctypes.byref(kpad))
    _check(rc, "fqo_plan_xw")
    return arrs[0], arrs[1], arrs[2], arrs[3], kp.value, kpad.value


def flatten_weights_split(W, src, rep_w, bits):
    """Weights with their own channels split (equal shares).  Returns (Wq int8 [N, Kpad], s_w)."""
    W = _f32(W)
    N, K = W.shape
    src = np.ascontiguousarray(src, dtype=np.int32)
    rep_w = np.ascontiguousarray(rep_w, dtype=np.int32)
    out = np.empty((N, src.shape[0]), dtype=np.int8)
    s_w = ctypes.c_float(0)
    rc = lib().fqo_flatten_weights_split(_p(W, ctypes.c_float), N, K, _p(src, ctypes.c_int32),
                                         _p(rep_w, ctypes.c_int32), src.shape[0], bits, _p(out, ctypes.c_int8),
                                         ctypes.byref(s_w))
    _check(rc, "fqo_flatten_weights_split")
    return out, np.float32(s_w.value)


def act_absmax_peel(X, T) -> np.float32:
    X = _f32(X)
    M, K = X.shape
    return np.float32(lib().fqo_act_absmax_peel(_p(X, ctypes.c_float), M, K, K, ctypes.c_float(T)))


def flatten_quant_act_peel(X, src, ord_, bits, T, a_prime):
    """Eq. 3 as printed + Eq. 1.  Returns (Xq int8 [M, Kpad], s_x)."""
    X = _f32(X)
    M, K = X.shape
    src = np.ascontiguousarray(src, dtype=np.int32)
    ord_ = np.ascontiguousarray(ord_, dtype=np.int32)
    out = np.empty((M, src.shape[0]), dtype=np.int8)
    s_x = ctypes.c_float(0)
    rc = lib().fqo_flatten_quant_act_peel(_p(X, ctypes.c_float), M, K, K, _p(src, ctypes.c_int32),
                                          _p(ord_, ctypes.c_int32), src.shape[0], bits, ctypes.c_float(T),
                                          ctypes.c_float(a_prime), _p(out, ctypes.c_int8), ctypes.byref(s_x))
    _check(rc, "fqo_flatten_quant_act_peel")
    return out, np.float32(s_x.value)


def dequant_bias(acc, s_x, s_w, bias):
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    rows, N = acc.shape
    bias = _f32(bias)
    assert bias.shape == (N,)
    out = np.empty((rows, N), dtype=np.float64)
    lib().fqo_dequant_bias(_p(acc, ctypes.c_int32), rows, N, ctypes.c_float(s_x), ctypes.c_float(s_w),
                           _p(bias, ctypes.c_float), _p(out, ctypes.c_double))
    return out


def dequant_out(acc, s_x, s_w, out_dtype, bias=None):
    """The layer's output as stored: fl32(fl32(acc) * fl32(s_x * s_w)) (+ bias, one more fp32 rounding)
    rounded to nearest-even to out_dtype in {"f32", "f16", "bf16"}.  Returns float32 values for "f32" and
    the uint16 bit patterns for the two 16-bit types, shaped like acc [rows, N]."""
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    rows, N = acc.shape
    code = {"f32": 0, "f16": 1, "bf16": 2}[out_dtype]
    out = np.empty((rows, N), dtype=np.float32 if code == 0 else np.uint16)
    pb = None
    if bias is not None:
        bias = _f32(bias)
        assert bias.shape == (N,)
        pb = _p(bias, ctypes.c_float)
    rc = lib().fqo_dequant_out(_p(acc, ctypes.c_int32), rows, N, ctypes.c_float(s_x), ctypes.c_float(s_w), pb, code,
                               out.ctypes.data_as(ctypes.c_void_p))
    _check(rc, "fqo_dequant_out")
    return out


def pack_e3m2(q):
    """4-bit values as packed 6-bit E3M2 codes: int8 [rows, Kpad] -> uint8 [rows, Kpad * 3 / 4]."""
    q = np.ascontiguousarray(q, dtype=np.int8)
    rows, Kpad = q.shape
    out = np.empty((rows, Kpad * 3 // 4), dtype=np.uint8)
    rc = lib().fqo_pack_e3m2(_p(q, ctypes.c_int8), ctypes.c_longlong(rows), Kpad, _p(out, ctypes.c_uint8))
    _check(rc, "fqo_pack_e3m2")
    return out


def pack_e3m2_blocked(q):
    """The same codes in the layout of the 6-bit GEMM: int8 [rows, Kpad] (Kpad a multiple of 128) -> uint8
    [Kpad / 128, rows, 96].  Block t holds 96 bytes for every row: two 48-byte groups (codes 128 t + 64 s ..
    + 63, s = 0, 1).  The 24-byte stream of each 32-code unit a of a group is split into its first 16 bytes
    X_a and last 8 bytes Y_a, and the group is stored X_a Y_a Y_b X_b with (a, b) = (0, 1) in rows whose
    index has bit 4 clear and (1, 0) in rows with bit 4 set."""
    q = np.ascontiguousarray(q, dtype=np.int8)
    rows, Kpad = q.shape
    if Kpad % 128:
        raise ValueError("Kpad must be a multiple of 128")
    nb = Kpad // 128
    stream = pack_e3m2(q).reshape(rows, nb, 2, 2, 24)        # [row, block, group, unit, stream byte]
    out = np.empty((nb, rows, 96), dtype=np.uint8)
    for r in range(rows):
        a, b = (0, 1) if (r & 16) == 0 else (1, 0)
        for t in range(nb):
            for s in range(2):
                ua, ub = stream[r, t, s, a], stream[r, t, s, b]
                out[t, r, 48 * s:48 * s + 48] = np.concatenate([ua[:16], ua[16:], ub[16:], ub[:16]])
    return out


def unpack_e3m2(packed):
    """Decodes packed E3M2 codes by the format's definition: uint8 [rows, Kpad*3/4] -> float64 [rows, Kpad]."""
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    rows, rb = packed.shape
    Kpad = rb * 4 // 3
    out = np.empty((rows, Kpad), dtype=np.float64)
    rc = lib().fqo_unpack_e3m2(_p(packed, ctypes.c_uint8), ctypes.c_longlong(rows), Kpad, _p(out, ctypes.c_double))
    _check(rc, "fqo_unpack_e3m2")
    return out
