"""Buffer bookkeeping for one quantized linear layer: owns the device buffers the C ABI wants
(map, quantized weights, scales, workspace) and forwards to the fq_* calls.  No arithmetic."""
import numpy as np

from . import binding as B


class FqLinear:
    """Offline: plan from (chmax, T) and quantize/repeat W.  Online: forward(X) -> Y."""

    def __init__(self, W, chmax: np.ndarray, T: float, bits: int, device="cuda:0", align: int = 0):
        """align = 0 picks the flattened-width padding that makes every quantized row start on a
        128-byte boundary (128 channels for INT8, 256 for packed INT4; E3M2 storage is blocked by 128), which the
        GEMM's direct global-to-LDS copies want; any multiple of 32 (the paper's padding) is accepted
        (128 for E3M2 storage).  bits = 8, 4, or binding.FQ_BITS_I4_E3M2 (4-bit values held as 6-bit codes
        for the 6-bit matrix pipe)."""
        import torch
        self.torch = torch
        self.bits = bits
        self.N, self.K = W.shape
        if align == 0:
            align = {8: 128, 4: 256, B.FQ_BITS_I4_E3M2: 128}[bits]
        src, rep, self.Kprime, self.Kpad = B.fq_flatten_plan(chmax, T, align)
        self.src_host, self.rep_host = src, rep
        self.src = torch.from_numpy(src).to(device)
        self.rep = torch.from_numpy(rep).to(device)
        if bits == B.FQ_BITS_I4_E3M2:
            self.Wq = torch.empty((self.Kpad // 128, self.N, 96), dtype=torch.uint8, device=device)
        else:
            cols = self.Kpad if bits == 8 else self.Kpad // 2
            self.Wq = torch.empty((self.N, cols), dtype=torch.int8 if bits == 8 else torch.uint8, device=device)
        self.s_w = torch.empty(1, dtype=torch.float32, device=device)
        ws = torch.empty(B.fq_weights_workspace_bytes(self.K, self.Kpad), dtype=torch.uint8, device=device)
        B.fq_flatten_weights(W, self.src, bits, self.Wq, self.s_w, ws)
        self.device = device
        self._ws = None
        self._ws_M = 0

    def workspace(self, M: int):
        if self._ws is None or self._ws_M < M:
            nbytes = B.fq_linear_workspace_bytes(M, self.K, self.Kpad, self.bits)
            self._ws = self.torch.empty(nbytes, dtype=self.torch.uint8, device=self.device)
            self._ws_M = M
        return self._ws

    def forward(self, X, Y=None, out_dtype=None, absmax_in=None):
        M = X.shape[0]
        if Y is None:
            Y = self.torch.empty((M, self.N), dtype=out_dtype or self.torch.bfloat16, device=X.device)
        B.fq_linear(X, self.src, self.rep, self.Wq, self.s_w, self.bits, Y, self.workspace(M), absmax_in=absmax_in)
        return Y
