"""Helpers for the GPU parity tests: move the synthetic workloads' bytes to the device and back."""
import numpy as np
import torch

DEV = "cuda:0"


def to_dev(store: np.ndarray, dtype: str):
    """Storage array from fq_workloads.round_to_dtype -> device tensor of the matching torch dtype."""
    if dtype == "bf16":
        return torch.from_numpy(store.view(np.int16)).to(DEV).view(torch.bfloat16)
    if dtype == "f16":
        return torch.from_numpy(store).to(DEV)
    return torch.from_numpy(np.ascontiguousarray(store, dtype=np.float32)).to(DEV)


def dev_i32(a: np.ndarray):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(DEV)


def scalar(v: float):
    return torch.tensor([v], dtype=torch.float32, device=DEV)


def bytes_ws(n: int):
    return torch.empty(max(int(n), 16), dtype=torch.uint8, device=DEV)


def bf16_to_f64(t):
    return t.float().cpu().numpy().astype(np.float64)


def rel_err(got: np.ndarray, ref: np.ndarray):
    """Element-wise relative error with the denominator floored at 1e-3 * rms(ref), so that
    outputs near zero do not blow the ratio up."""
    floor = 1e-3 * float(np.sqrt(np.mean(ref.astype(np.float64) ** 2))) + 1e-300
    return np.abs(got - ref) / np.maximum(np.abs(ref), floor)


def bits16(t) -> np.ndarray:
    """Bit patterns of a 2-byte floating-point device tensor (bf16 or half) as uint16."""
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def bits32(t) -> np.ndarray:
    return t.contiguous().view(torch.int32).cpu().numpy().view(np.uint32)
