"""The entry point that allocates nothing: fq_flatten_quant_act_noalloc against fq_flatten_quant_act.

Same kernels, the workspace inside the library's device image instead of a caller-owned buffer: the
quantized bytes and the scale must be identical.  Two calls in a row, the second on a smaller input
(the shared array keeps the first call's contents), then a static-scale call; and the size limit."""
import numpy as np
import pytest
import torch

import fq_workloads as WL
import paper_2402_17985_amd as fq
from tests.gpu_util import DEV, bytes_ws, dev_i32, scalar, to_dev


def _both(L, bits, a_static=None):
    src, rep, kp, kpad = fq.fq_flatten_plan(L.chmax, L.T, 256)
    M, K = L.X.shape
    Xd = to_dev(L.X_store, L.spec.x_dtype)
    srcd, repd = dev_i32(src), dev_i32(rep)
    cols = kpad if bits == 8 else kpad // 2
    a_in = None if a_static is None else scalar(a_static)
    ref = torch.full((M, cols), 0x55, dtype=torch.uint8, device=DEV)
    s_ref = torch.zeros(1, dtype=torch.float32, device=DEV)
    fq.fq_flatten_quant_act(Xd, srcd, repd, bits, ref, s_ref, bytes_ws(fq.fq_act_workspace_bytes(K, kpad)), absmax_in=a_in)
    got = torch.full((M, cols), 0xAA, dtype=torch.uint8, device=DEV)
    s_got = torch.zeros(1, dtype=torch.float32, device=DEV)
    before = torch.cuda.memory_allocated()
    fq.fq_flatten_quant_act_noalloc(Xd, srcd, repd, bits, got, s_got, absmax_in=a_in)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    assert s_got.item() == s_ref.item()
    assert torch.equal(got, ref)
    return kpad


@pytest.mark.gpu
@pytest.mark.parametrize("bits", [8, 4])
def test_noalloc_equals_workspace_call_twice_then_smaller(bits):
    big = WL.make_layer(WL.CONFIGS["cfg3"], 0, M_override=1029, K_override=4096, N_override=8)
    small = WL.make_layer(WL.CONFIGS["cfg2"], 0, M_override=77, K_override=1024, N_override=8)
    print(f"[noalloc] bits={bits} big M=1029 K=4096, then small M=77 K=1024", flush=True)
    kpad_big = _both(big, bits)
    kpad_small = _both(small, bits)                 # smaller input: the array still holds the first call's values
    assert kpad_small < kpad_big
    _both(small, bits, a_static=small.T)            # static scale: no absmax pass, no clearing needed
    _both(big, bits)


def test_noalloc_rejects_sizes_beyond_the_builtin_scratch():
    """Checked on the host before anything touches a device: no GPU needed."""
    L = fq.lib()
    assert fq.fq_noalloc_scratch_bytes() == 1 << 20
    K, Kpad = 200000, 262144 - 256
    assert fq.fq_act_workspace_bytes(K, Kpad) > fq.fq_noalloc_scratch_bytes()
    fake = 0x10000            # never dereferenced: the call fails before any launch
    rc = L.fq_flatten_quant_act_noalloc(fake, fq.FQ_BF16, 4, K, K, fake, fake, 131072 - 256, 8, None, fake, fake, None)
    assert rc != 0            # Kpad at the accumulator bound still exceeds the scratch for this K
    assert b"scratch" in L.fq_last_error_string()
