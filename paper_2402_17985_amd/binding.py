"""Thin Python binding of libfq.so (include/fq.h).

Argument marshalling only: every step of the path runs in the HIP kernels behind the C ABI.
PyTorch tensors are used as device buffers (`data_ptr()`) and for the current stream; nothing is
computed in PyTorch.  There is no fallback: if libfq.so is missing, loading raises.
"""
import ctypes
import os
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfq.so")

FQ_F32, FQ_F16, FQ_BF16, FQ_I32 = 0, 1, 2, 3
FQ_OK = 0
ERR_NAMES = {1: "FQ_ERR_NULL", 2: "FQ_ERR_SHAPE", 3: "FQ_ERR_DTYPE", 4: "FQ_ERR_RANGE", 5: "FQ_ERR_ALIGN",
             6: "FQ_ERR_HIP", 7: "FQ_ERR_WORKSPACE"}

# every entry point include/fq.h declares
SYMBOLS = ["fq_last_error_string", "fq_version", "fq_flatten_plan", "fq_flatten_weights",
           "fq_weights_workspace_bytes", "fq_flatten_quant_act", "fq_act_workspace_bytes", "fq_gemm_i8",
           "fq_gemm_i4", "fq_linear", "fq_linear_workspace_bytes", "fq_gemm_bf16", "fq_gemm_select",
           "fq_threshold_boxplot", "fq_smooth_scales", "fq_channel_absmax", "fq_bmm_i8", "fq_bmm_i4",
           "fq_flatten_plan_xw", "fq_flatten_weights_split", "fq_flatten_quant_act_peel",
           "fq_gemm_i8_bias", "fq_gemm_i4_bias", "fq_linear_bias", "fq_linear_fused_a_i8", "fq_gemm_i4_e3m2",
           "fq_flatten_quant_act_noalloc", "fq_noalloc_scratch_bytes",
           # include/fq_peak.h: measurement hooks
           "fq_peak_mfma", "fq_peak_copy", "fq_peak_gemm_ticks", "fq_peak_wall_clock_khz"]
FQ_PEAK_I8, FQ_PEAK_BF16, FQ_PEAK_E3M2, FQ_PEAK_I8_NIBBLES = 0, 1, 2, 3
FQ_BITS_I4_E3M2 = 6   # the 4-bit quantizer with its values stored as 6-bit E3M2 codes


class FqError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"{ERR_NAMES.get(code, code)}: {msg}")
        self.code = code


_lib = None


def lib() -> ctypes.CDLL:
    """Load libfq.so (built in-tree by paper_2402_17985_amd/build.py).  Raises if it is absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(f"{LIB_PATH} not found: build it with `python -m paper_2402_17985_amd.build` "
                                "(there is no CPU or PyTorch fallback)")
    L = ctypes.CDLL(LIB_PATH)
    c_int, c_float, c_size_t, vp = ctypes.c_int, ctypes.c_float, ctypes.c_size_t, ctypes.c_void_p
    L.fq_last_error_string.restype = ctypes.c_char_p
    L.fq_last_error_string.argtypes = []
    L.fq_version.restype = c_int
    L.fq_gemm_select.argtypes = [c_int]
    L.fq_flatten_plan.argtypes = [vp, c_int, c_float, c_int, vp, vp, c_int, ctypes.POINTER(c_int),
                                  ctypes.POINTER(c_int)]
    L.fq_threshold_boxplot.argtypes = [vp, c_int, c_float, ctypes.POINTER(c_float)]
    L.fq_smooth_scales.argtypes = [vp, vp, c_int, c_float, vp]
    L.fq_flatten_plan_xw.argtypes = [vp, c_float, vp, c_float, c_int, c_int, vp, vp, vp, vp, c_int,
                                     ctypes.POINTER(c_int), ctypes.POINTER(c_int)]
    L.fq_flatten_weights_split.argtypes = [vp, c_int, c_int, c_int, c_int, vp, vp, c_int, c_int, vp, vp, vp, c_size_t, vp]
    L.fq_flatten_quant_act_peel.argtypes = [vp, c_int, c_int, c_int, c_int, vp, vp, c_int, c_int, c_float, vp, vp, vp,
                                            vp, c_size_t, vp]
    L.fq_channel_absmax.argtypes = [vp, c_int, c_int, c_int, c_int, c_int, vp, vp]
    L.fq_flatten_weights.argtypes = [vp, c_int, c_int, c_int, c_int, vp, c_int, c_int, vp, vp, vp, c_size_t, vp]
    L.fq_weights_workspace_bytes.restype = c_size_t
    L.fq_weights_workspace_bytes.argtypes = [c_int, c_int]
    L.fq_flatten_quant_act.argtypes = [vp, c_int, c_int, c_int, c_int, vp, vp, c_int, c_int, vp, vp, vp, vp,
                                       c_size_t, vp]
    L.fq_flatten_quant_act_noalloc.argtypes = [vp, c_int, c_int, c_int, c_int, vp, vp, c_int, c_int, vp, vp, vp, vp]
    L.fq_noalloc_scratch_bytes.restype = c_size_t
    L.fq_noalloc_scratch_bytes.argtypes = []
    L.fq_peak_mfma.argtypes = [c_int, vp, c_size_t, c_int, ctypes.c_longlong, vp, vp, vp]
    L.fq_peak_copy.argtypes = [vp, vp, c_size_t, vp]
    L.fq_peak_gemm_ticks.argtypes = [vp]
    L.fq_peak_wall_clock_khz.argtypes = []
    L.fq_act_workspace_bytes.restype = c_size_t
    L.fq_act_workspace_bytes.argtypes = [c_int, c_int]
    for f in (L.fq_gemm_i8, L.fq_gemm_i4):
        f.argtypes = [vp, vp, c_int, c_int, c_int, vp, vp, vp, c_int, c_int, vp]
    for f in (L.fq_bmm_i8, L.fq_bmm_i4):
        f.argtypes = [vp, vp, c_int, c_int, c_int, c_int, ctypes.c_longlong, ctypes.c_longlong, vp, vp, vp, c_int,
                      c_int, ctypes.c_longlong, vp]
    for f in (L.fq_gemm_i8_bias, L.fq_gemm_i4_bias, L.fq_gemm_i4_e3m2):
        f.argtypes = [vp, vp, c_int, c_int, c_int, vp, vp, vp, vp, c_int, c_int, vp]
    L.fq_linear_fused_a_i8.argtypes = [vp, c_int, c_int, c_int, c_int, vp, vp, c_int, vp, vp, vp, c_int, vp, vp, c_int, c_int,
                                       vp, c_size_t, vp]
    L.fq_linear_bias.argtypes = [vp, c_int, c_int, c_int, c_int, vp, vp, c_int, vp, vp, vp, c_int, c_int, vp, vp,
                                 c_int, c_int, vp, c_size_t, vp]
    L.fq_linear.argtypes = [vp, c_int, c_int, c_int, c_int, vp, vp, c_int, vp, vp, c_int, c_int, vp, vp, c_int,
                            c_int, vp, c_size_t, vp]
    L.fq_linear_workspace_bytes.restype = c_size_t
    L.fq_linear_workspace_bytes.argtypes = [c_int, c_int, c_int, c_int]
    L.fq_gemm_bf16.argtypes = [vp, vp, c_int, c_int, c_int, vp, c_int, vp]
    for name in SYMBOLS:
        getattr(L, name)
    _lib = L
    return L


def _check(rc: int):
    if rc != FQ_OK:
        raise FqError(rc, lib().fq_last_error_string().decode())


def _torch():
    import torch
    return torch


def _dtype_code(t) -> int:
    torch = _torch()
    return {torch.float32: FQ_F32, torch.float16: FQ_F16, torch.bfloat16: FQ_BF16, torch.int32: FQ_I32}[t.dtype]


def _stream(stream) -> int:
    if stream is None:
        return _torch().cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _dev2d(t, name):
    if not t.is_cuda:
        raise ValueError(f"{name} must be a device tensor")
    if t.dim() != 2 or t.stride(1) != 1:
        raise ValueError(f"{name} must be 2-D with a contiguous last dimension")
    return t


# ------------------------------------------------------------------------------------------
# entry points (same names as the C ABI)
# ------------------------------------------------------------------------------------------
def fq_version() -> int:
    return lib().fq_version()


def fq_gemm_select(variant: int) -> None:
    _check(lib().fq_gemm_select(variant))


def fq_flatten_plan(chmax: np.ndarray, T: float, align: int = 32) -> Tuple[np.ndarray, np.ndarray, int, int]:
    """Host call.  Returns (src_idx int32 [Kpad], rep int32 [Kpad], Kprime, Kpad)."""
    chmax = np.ascontiguousarray(chmax, dtype=np.float32)
    K = chmax.shape[0]
    kp, kpad = ctypes.c_int(0), ctypes.c_int(0)
    _check(lib().fq_flatten_plan(chmax.ctypes.data, K, T, align, None, None, 0, ctypes.byref(kp), ctypes.byref(kpad)))
    src = np.empty(kpad.value, dtype=np.int32)
    rep = np.empty(kpad.value, dtype=np.int32)
    _check(lib().fq_flatten_plan(chmax.ctypes.data, K, T, align, src.ctypes.data, rep.ctypes.data, kpad.value,
                                 ctypes.byref(kp), ctypes.byref(kpad)))
    return src, rep, kp.value, kpad.value


def fq_flatten_plan_xw(chmax_x: np.ndarray, T_x: float, chmax_w: Optional[np.ndarray] = None, T_w: float = 1.0,
                       align: int = 32):
    """Host call.  Returns (src_idx, rep_x, rep_w, ord, Kprime, Kpad), int32 arrays of Kpad entries."""
    chmax_x = np.ascontiguousarray(chmax_x, dtype=np.float32)
    K = chmax_x.shape[0]
    cw = None if chmax_w is None else np.ascontiguousarray(chmax_w, dtype=np.float32)
    if cw is not None and cw.shape != chmax_x.shape:
        raise ValueError("chmax_x and chmax_w must have the same length")
    pw = None if cw is None else cw.ctypes.data
    kp, kpad = ctypes.c_int(0), ctypes.c_int(0)
    _check(lib().fq_flatten_plan_xw(chmax_x.ctypes.data, T_x, pw, T_w, K, align, None, None, None, None, 0,
                                    ctypes.byref(kp), ctypes.byref(kpad)))
    arrs = [np.empty(kpad.value, dtype=np.int32) for _ in range(4)]
    _check(lib().fq_flatten_plan_xw(chmax_x.ctypes.data, T_x, pw, T_w, K, align, *[a.ctypes.data for a in arrs],
                                    kpad.value, ctypes.byref(kp), ctypes.byref(kpad)))
    return arrs[0], arrs[1], arrs[2], arrs[3], kp.value, kpad.value


def fq_threshold_boxplot(chmax: np.ndarray, beta: float = 1.3) -> float:
    """Host call (Eq. 6-7).  Returns T as a Python float holding an fp32 value."""
    chmax = np.ascontiguousarray(chmax, dtype=np.float32)
    T = ctypes.c_float(0)
    _check(lib().fq_threshold_boxplot(chmax.ctypes.data, chmax.shape[0], beta, ctypes.byref(T)))
    return float(T.value)


def fq_smooth_scales(chmax_x: np.ndarray, chmax_w: np.ndarray, alpha: float = 0.5) -> np.ndarray:
    """Host call (Eq. 5).  Returns the fp32 smoothing factors s [K]."""
    chmax_x = np.ascontiguousarray(chmax_x, dtype=np.float32)
    chmax_w = np.ascontiguousarray(chmax_w, dtype=np.float32)
    if chmax_x.shape != chmax_w.shape:
        raise ValueError("chmax_x and chmax_w must have the same length")
    out = np.empty(chmax_x.shape[0], dtype=np.float32)
    _check(lib().fq_smooth_scales(chmax_x.ctypes.data, chmax_w.ctypes.data, chmax_x.shape[0], alpha, out.ctypes.data))
    return out


def fq_channel_absmax(X, chmax, accumulate: bool = False, stream=None) -> None:
    """chmax (fp32 [K], device) = per-channel max |X|, or the running maximum when accumulate is set."""
    _dev2d(X, "X")
    M, K = X.shape
    if chmax.numel() != K or _dtype_code(chmax) != FQ_F32 or not chmax.is_contiguous():
        raise ValueError("chmax must be a contiguous fp32 tensor of K elements")
    _check(lib().fq_channel_absmax(X.data_ptr(), _dtype_code(X), M, K, X.stride(0), int(bool(accumulate)),
                                   chmax.data_ptr(), _stream(stream)))


def fq_weights_workspace_bytes(K: int, Kpad: int) -> int:
    return lib().fq_weights_workspace_bytes(K, Kpad)


def fq_act_workspace_bytes(K: int, Kpad: int) -> int:
    return lib().fq_act_workspace_bytes(K, Kpad)


def fq_linear_workspace_bytes(M: int, K: int, Kpad: int, bits: int) -> int:
    return lib().fq_linear_workspace_bytes(M, K, Kpad, bits)


def fq_flatten_weights(W, src_idx, bits: int, Wq_out, s_w_out, workspace, stream=None) -> None:
    _dev2d(W, "W")
    N, K = W.shape
    Kpad = src_idx.numel()
    _check(lib().fq_flatten_weights(W.data_ptr(), _dtype_code(W), N, K, W.stride(0), src_idx.data_ptr(), Kpad, bits,
                                    Wq_out.data_ptr(), s_w_out.data_ptr(), workspace.data_ptr(),
                                    workspace.numel() * workspace.element_size(), _stream(stream)))


def fq_flatten_weights_split(W, src_idx, rep_w, bits: int, Wq_out, s_w_out, workspace, stream=None) -> None:
    _dev2d(W, "W")
    N, K = W.shape
    Kpad = src_idx.numel()
    _check(lib().fq_flatten_weights_split(W.data_ptr(), _dtype_code(W), N, K, W.stride(0), src_idx.data_ptr(),
                                          rep_w.data_ptr(), Kpad, bits, Wq_out.data_ptr(), s_w_out.data_ptr(),
                                          workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                          _stream(stream)))


def fq_flatten_quant_act_peel(X, src_idx, ord, bits: int, T: float, Xq_out, s_x_out, workspace, absmax_in=None,
                              stream=None) -> None:
    _dev2d(X, "X")
    M, K = X.shape
    Kpad = src_idx.numel()
    _check(lib().fq_flatten_quant_act_peel(X.data_ptr(), _dtype_code(X), M, K, X.stride(0), src_idx.data_ptr(),
                                           ord.data_ptr(), Kpad, bits, T, _ptr(absmax_in), Xq_out.data_ptr(),
                                           s_x_out.data_ptr(), workspace.data_ptr(),
                                           workspace.numel() * workspace.element_size(), _stream(stream)))


def fq_flatten_quant_act(X, src_idx, rep, bits: int, Xq_out, s_x_out, workspace, absmax_in=None, stream=None) -> None:
    _dev2d(X, "X")
    M, K = X.shape
    Kpad = src_idx.numel()
    _check(lib().fq_flatten_quant_act(X.data_ptr(), _dtype_code(X), M, K, X.stride(0), src_idx.data_ptr(),
                                      rep.data_ptr(), Kpad, bits, _ptr(absmax_in), Xq_out.data_ptr(),
                                      s_x_out.data_ptr(), workspace.data_ptr(),
                                      workspace.numel() * workspace.element_size(), _stream(stream)))


def fq_noalloc_scratch_bytes() -> int:
    return int(lib().fq_noalloc_scratch_bytes())


def fq_flatten_quant_act_noalloc(X, src_idx, rep, bits: int, Xq_out, s_x_out, absmax_in=None, stream=None) -> None:
    """fq_flatten_quant_act with the workspace inside the library's device image (nothing is allocated)."""
    _dev2d(X, "X")
    M, K = X.shape
    Kpad = src_idx.numel()
    _check(lib().fq_flatten_quant_act_noalloc(X.data_ptr(), _dtype_code(X), M, K, X.stride(0), src_idx.data_ptr(),
                                              rep.data_ptr(), Kpad, bits, _ptr(absmax_in), Xq_out.data_ptr(),
                                              s_x_out.data_ptr(), _stream(stream)))


def fq_peak_mfma(kind: int, operands, blocks: int, iters: int, ticks_out, sink, stream=None) -> None:
    """MFMA-only issue loop (include/fq_peak.h).  operands: a device tensor of >= 64 KiB, or None for zeros."""
    nbytes = 0 if operands is None else operands.numel() * operands.element_size()
    _check(lib().fq_peak_mfma(kind, _ptr(operands), nbytes, blocks, iters, _ptr(ticks_out), sink.data_ptr(),
                              _stream(stream)))


def fq_peak_gemm_ticks(ticks) -> None:
    """ticks: int64 device tensor [2] the GEMM kernels launched from this thread add their clock ticks to, or None."""
    _check(lib().fq_peak_gemm_ticks(_ptr(ticks)))


def fq_peak_wall_clock_khz() -> int:
    return int(lib().fq_peak_wall_clock_khz())


def fq_peak_copy(src, dst, stream=None) -> None:
    """Plain device copy of src into dst (same byte size, a multiple of 16)."""
    nbytes = src.numel() * src.element_size()
    assert nbytes == dst.numel() * dst.element_size()
    _check(lib().fq_peak_copy(src.data_ptr(), dst.data_ptr(), nbytes, _stream(stream)))


def _gemm(fn, Xq, Wq, M, N, Kpad, s_x, s_w, Y, stream):
    _dev2d(Y, "Y")
    _check(fn(Xq.data_ptr(), Wq.data_ptr(), M, N, Kpad, _ptr(s_x), _ptr(s_w), Y.data_ptr(), _dtype_code(Y),
              Y.stride(0), _stream(stream)))


def fq_gemm_i8(Xq, Wq, s_x, s_w, Y, stream=None) -> None:
    """Xq int8 [M, Kpad], Wq int8 [N, Kpad] -> Y [M, N] (f32/f16/bf16, or int32 raw accumulators)."""
    M, Kpad = Xq.shape
    N = Wq.shape[0]
    _gemm(lib().fq_gemm_i8, Xq, Wq, M, N, Kpad, s_x, s_w, Y, stream)


def _gemm_bias(fn, Xq, Wq, M, N, Kpad, s_x, s_w, bias, Y, stream):
    _dev2d(Y, "Y")
    if bias is not None and (bias.numel() != N or _dtype_code(bias) != FQ_F32 or not bias.is_contiguous()):
        raise ValueError("bias must be a contiguous fp32 tensor of N elements")
    _check(fn(Xq.data_ptr(), Wq.data_ptr(), M, N, Kpad, _ptr(s_x), _ptr(s_w), _ptr(bias), Y.data_ptr(), _dtype_code(Y),
              Y.stride(0), _stream(stream)))


def fq_gemm_i8_bias(Xq, Wq, s_x, s_w, bias, Y, stream=None) -> None:
    M, Kpad = Xq.shape
    _gemm_bias(lib().fq_gemm_i8_bias, Xq, Wq, M, Wq.shape[0], Kpad, s_x, s_w, bias, Y, stream)


def fq_gemm_i4_bias(Xq, Wq, s_x, s_w, bias, Y, stream=None) -> None:
    M, half = Xq.shape
    _gemm_bias(lib().fq_gemm_i4_bias, Xq, Wq, M, Wq.shape[0], 2 * half, s_x, s_w, bias, Y, stream)


def fq_gemm_i4_e3m2(Xq, Wq, s_x, s_w, bias, Y, stream=None) -> None:
    """Xq uint8 [Kpad / 128, M, 96], Wq uint8 [Kpad / 128, N, 96] (k-blocked 6-bit E3M2 codes of 4-bit values)
    -> Y [M, N]."""
    if Xq.dim() != 3 or Wq.dim() != 3 or Xq.shape[2] != 96 or Wq.shape[2] != 96 or Xq.shape[0] != Wq.shape[0]:
        raise ValueError("E3M2 operands are [Kpad / 128, rows, 96] byte arrays")
    if not (Xq.is_contiguous() and Wq.is_contiguous()):
        raise ValueError("E3M2 operands must be contiguous")
    _gemm_bias(lib().fq_gemm_i4_e3m2, Xq, Wq, Xq.shape[1], Wq.shape[1], 128 * Xq.shape[0], s_x, s_w, bias, Y, stream)


def fq_linear_bias(X, src_idx, rep, Wq, s_w, bias, bits: int, Y, workspace, absmax_in=None, stream=None) -> None:
    _dev2d(X, "X")
    _dev2d(Y, "Y")
    M, K = X.shape
    Kpad = src_idx.numel()
    N = Wq.shape[1] if Wq.dim() == 3 else Wq.shape[0]      # E3M2 weights are [Kpad / 128, N, 96]
    if bias is not None and (bias.numel() != N or _dtype_code(bias) != FQ_F32 or not bias.is_contiguous()):
        raise ValueError("bias must be a contiguous fp32 tensor of N elements")
    _check(lib().fq_linear_bias(X.data_ptr(), _dtype_code(X), M, K, X.stride(0), src_idx.data_ptr(), rep.data_ptr(),
                                Kpad, Wq.data_ptr(), s_w.data_ptr(), _ptr(bias), N, bits, _ptr(absmax_in), Y.data_ptr(),
                                _dtype_code(Y), Y.stride(0), workspace.data_ptr(),
                                workspace.numel() * workspace.element_size(), _stream(stream)))


def fq_linear_fused_a_i8(X, src_idx, rep, Wq, s_w, Y, workspace, bias=None, absmax_in=None, stream=None) -> None:
    """The INT8 layer with flatten + quantize fused into the GEMM's A-operand load: X bf16 [M, K], Wq int8 [N, Kpad]
    -> Y [M, N]; workspace of fq_act_workspace_bytes(K, Kpad) bytes."""
    _dev2d(X, "X")
    _dev2d(Y, "Y")
    M, K = X.shape
    Kpad = src_idx.numel()
    N = Wq.shape[0]
    if bias is not None and (bias.numel() != N or _dtype_code(bias) != FQ_F32 or not bias.is_contiguous()):
        raise ValueError("bias must be a contiguous fp32 tensor of N elements")
    _check(lib().fq_linear_fused_a_i8(X.data_ptr(), _dtype_code(X), M, K, X.stride(0), src_idx.data_ptr(), rep.data_ptr(),
                                      Kpad, Wq.data_ptr(), _ptr(s_w), _ptr(bias), N, _ptr(absmax_in), Y.data_ptr(),
                                      _dtype_code(Y), Y.stride(0), workspace.data_ptr(),
                                      workspace.numel() * workspace.element_size(), _stream(stream)))


def fq_gemm_i4(Xq, Wq, s_x, s_w, Y, stream=None) -> None:
    """Xq uint8 [M, Kpad/2], Wq uint8 [N, Kpad/2] (packed nibbles) -> Y [M, N]."""
    M, half = Xq.shape
    N = Wq.shape[0]
    _gemm(lib().fq_gemm_i4, Xq, Wq, M, N, 2 * half, s_x, s_w, Y, stream)


def _bmm(fn, Aq, Bq, Kpad, s_a, s_b, Y, stream):
    for t, name in ((Aq, "Aq"), (Bq, "Bq"), (Y, "Y")):
        if not t.is_cuda or t.dim() != 3 or t.stride(2) != 1:
            raise ValueError(f"{name} must be a 3-D device tensor with a contiguous last dimension")
    batch, M, rowbytes = Aq.shape
    N = Bq.shape[1]
    if Bq.shape[0] != batch or Bq.shape[2] != rowbytes or Y.shape != (batch, M, N):
        raise ValueError("shape mismatch between Aq, Bq and Y")
    if Aq.stride(1) != rowbytes or Bq.stride(1) != rowbytes:
        raise ValueError("operand rows must be dense")
    _check(fn(Aq.data_ptr(), Bq.data_ptr(), batch, M, N, Kpad, Aq.stride(0), Bq.stride(0), _ptr(s_a), _ptr(s_b),
              Y.data_ptr(), _dtype_code(Y), Y.stride(1), Y.stride(0), _stream(stream)))


def fq_bmm_i8(Aq, Bq, s_a, s_b, Y, stream=None) -> None:
    """Aq int8 [batch, M, Kpad], Bq int8 [batch, N, Kpad] -> Y [batch, M, N]."""
    _bmm(lib().fq_bmm_i8, Aq, Bq, Aq.shape[2], s_a, s_b, Y, stream)


def fq_bmm_i4(Aq, Bq, s_a, s_b, Y, stream=None) -> None:
    """Aq uint8 [batch, M, Kpad/2], Bq uint8 [batch, N, Kpad/2] (packed nibbles) -> Y [batch, M, N]."""
    _bmm(lib().fq_bmm_i4, Aq, Bq, 2 * Aq.shape[2], s_a, s_b, Y, stream)


def fq_linear(X, src_idx, rep, Wq, s_w, bits: int, Y, workspace, absmax_in=None, stream=None) -> None:
    _dev2d(X, "X")
    _dev2d(Y, "Y")
    M, K = X.shape
    Kpad = src_idx.numel()
    N = Wq.shape[1] if Wq.dim() == 3 else Wq.shape[0]      # E3M2 weights are [Kpad / 128, N, 96]
    _check(lib().fq_linear(X.data_ptr(), _dtype_code(X), M, K, X.stride(0), src_idx.data_ptr(), rep.data_ptr(), Kpad,
                           Wq.data_ptr(), s_w.data_ptr(), N, bits, _ptr(absmax_in), Y.data_ptr(), _dtype_code(Y),
                           Y.stride(0), workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                           _stream(stream)))


def fq_gemm_bf16(X, W, Y, stream=None) -> None:
    _dev2d(X, "X")
    _dev2d(W, "W")
    _dev2d(Y, "Y")
    M, K = X.shape
    N = W.shape[0]
    if X.stride(0) != K or W.stride(0) != K:
        raise ValueError("fq_gemm_bf16 needs densely packed rows")
    _check(lib().fq_gemm_bf16(X.data_ptr(), W.data_ptr(), M, N, K, Y.data_ptr(), Y.stride(0), _stream(stream)))
