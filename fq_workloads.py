"""Seeded synthetic workloads for the FlattenQuant linear-layer hot path.

This module only SYNTHESISES INPUTS (activations with outlier channels, weights, the
"calibrated" per-channel maxima and the truncation threshold T handed to the planner).  It
holds none of the method's arithmetic (no plan, no quantizer, no GEMM) and is the one module
the GPU tests/bench and the CPU oracle's tests both import, so that both sides see the same
bytes.  The paper measured on OPT activations from public datasets (Sec. 5.1); those are
replaced here by Gaussian activations in which a small fraction of channels is scaled up
20-100x, the outlier structure the paper describes in Sec. 3.1.

Generator: NumPy default_rng (PCG64) seeded with (config seed, layer index); draw order is
X, outlier channel indices, outlier factors, W.  Outlier channels are scaled in fp32, then the
tensor is rounded (nearest-even) to the layer's storage dtype.
"""
from dataclasses import dataclass, field
from typing import Optional, Tuple

import numpy as np


# ------------------------------------------------------------------------------------------
# dtype plumbing (bit-level only)
# ------------------------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bfloat16 (nearest-even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns exactly to fp32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_dtype(x: np.ndarray, dtype: str) -> Tuple[np.ndarray, np.ndarray]:
    """Returns (storage array as handed to the GPU, the same values widened exactly to fp32)."""
    if dtype == "f32":
        x = np.ascontiguousarray(x, dtype=np.float32)
        return x, x
    if dtype == "bf16":
        bits = f32_to_bf16_bits(x)
        return bits, bf16_bits_to_f32(bits)
    if dtype == "f16":
        h = np.ascontiguousarray(x, dtype=np.float32).astype(np.float16)
        return h, h.astype(np.float32)
    raise ValueError(dtype)


# ------------------------------------------------------------------------------------------
# workload table
# ------------------------------------------------------------------------------------------
@dataclass(frozen=True)
class LayerSpec:
    name: str
    M: int
    K: int
    N: int
    bits: int
    x_dtype: str = "bf16"
    w_dtype: str = "bf16"
    w_std: Optional[float] = None            # None -> 1/sqrt(K)
    outlier_frac: float = 0.005              # fraction of channels scaled up
    outlier_fixed: Optional[Tuple[Tuple[int, float], ...]] = None   # explicit (channel, factor)
    factor_range: Tuple[float, float] = (10.0, 100.0)
    t_rule: str = "3xmedian"                 # see threshold()
    t_value: Optional[float] = None          # the threshold itself (rule "value")


@dataclass(frozen=True)
class Config:
    name: str
    seed: int
    layers: Tuple[LayerSpec, ...]
    note: str = ""


_FIXED1 = ((3, 8.0), (50, 16.0), (101, 32.0), (200, 64.0))

CONFIGS = {
    # tiny; as written the threshold exceeds every channel maximum, so nothing is flattened
    "cfg1": Config("cfg1", 0, (LayerSpec("tiny", 16, 256, 256, 8, "f32", "f32", 0.02, 0.0, _FIXED1,
                                         t_rule="2xp99.9_abs"),)),
    # same tensors with T = 8 so that the four scaled channels are flattened
    "cfg1b": Config("cfg1b", 0, (LayerSpec("tiny_T8", 16, 256, 256, 8, "f32", "f32", 0.02, 0.0, _FIXED1,
                                           t_rule="value", t_value=8.0),)),
    "cfg2": Config("cfg2", 1, (LayerSpec("qkv", 2048, 4096, 4096, 8, t_rule="3xp99_chmax"),)),
    "cfg3": Config("cfg3", 2, (LayerSpec("ffn1", 8192, 4096, 11008, 4, t_rule="top15pct"),
                               LayerSpec("ffn2", 8192, 11008, 4096, 4, t_rule="top15pct"))),
    # INT8 companion at the metric's M=8192 LLaMA-7B shape
    "cfg3i8": Config("cfg3i8", 2, (LayerSpec("proj", 8192, 4096, 4096, 8, t_rule="top15pct"),)),
    "cfg4": Config("cfg4", 3, tuple(
        LayerSpec(n, 8192, k, nn, b, outlier_frac=0.01, factor_range=(20.0, 200.0))
        for (n, k, nn, b) in (("qkv", 5120, 15360, 8), ("out", 5120, 5120, 8),
                              ("fc1", 5120, 20480, 4), ("fc2", 20480, 5120, 4)))),
    "cfg5": Config("cfg5", 4, tuple(
        LayerSpec(n, 16384, k, nn, b, outlier_frac=0.003, factor_range=(10.0, 300.0))
        for (n, k, nn, b) in (("qkv", 8192, 24576, 8), ("out", 8192, 8192, 8),
                              ("ffn1", 8192, 22016, 4), ("ffn2", 22016, 8192, 4)))),
    # the shape of the paper's operator measurement (Table 5): 8 x 2048 tokens, 4096 -> 4096, about 1024
    # expanded channels.  The thresholds are literals, found once for these seeded tensors as the smallest fp32
    # value at which the flattened width grows by at most 1024 channels; the full-size test checks that count
    # through the planner.
    "cfgP": Config("cfgP", 5, tuple(
        LayerSpec(n, 16384, 4096, 4096, b, outlier_frac=0.01, factor_range=(10.0, 100.0), t_rule="value", t_value=t)
        for (n, b, t) in (("table5_int8", 8, 7.0), ("table5_int4", 4, 6.888889312744141)))),
}


@dataclass
class Layer:
    spec: LayerSpec
    X_store: np.ndarray          # storage-dtype array (uint16 bit patterns for bf16)
    X: np.ndarray                # the same values, fp32
    W_store: np.ndarray
    W: np.ndarray
    chmax: np.ndarray            # fp32 [K], max_i |X[i, j]|
    T: float
    outlier_idx: np.ndarray = field(default_factory=lambda: np.zeros(0, np.int64))


def threshold(rule: str, X: np.ndarray, chmax: np.ndarray, value: Optional[float] = None) -> float:
    """The configs' threshold rules (inputs to the planner, not part of the method)."""
    K = chmax.shape[0]
    if rule == "value":
        return float(np.float32(value))
    if rule == "2xp99.9_abs":
        return float(np.float32(2.0 * np.percentile(np.abs(X).astype(np.float64), 99.9)))
    if rule == "3xp99_chmax":
        return float(np.float32(3.0 * np.percentile(chmax.astype(np.float64), 99.0)))
    if rule == "3xmedian":
        return float(np.float32(3.0 * np.median(chmax.astype(np.float64))))
    if rule == "top15pct":
        # the (floor(0.15 K) + 1)-th largest channel maximum: exactly floor(0.15 K) channels
        # exceed it (barring ties), i.e. at most 15 % of channels are flattened
        k = int(np.floor(0.15 * K))
        return float(np.sort(chmax)[::-1][k])
    raise ValueError(rule)


def make_layer(cfg: Config, index: int, M_override: Optional[int] = None,
               K_override: Optional[int] = None, N_override: Optional[int] = None) -> Layer:
    """Generate layer `index` of `cfg`.  The overrides shrink a workload for parity tests while
    keeping its recipe (distribution, outlier fraction, threshold rule)."""
    spec = cfg.layers[index]
    if M_override or K_override or N_override:
        spec = LayerSpec(**{**spec.__dict__, "M": M_override or spec.M, "K": K_override or spec.K,
                            "N": N_override or spec.N})
    rng = np.random.default_rng([cfg.seed, index])
    M, K, N = spec.M, spec.K, spec.N
    X = rng.standard_normal((M, K), dtype=np.float32)
    if spec.outlier_fixed is not None:
        idx = np.array([c for c, _ in spec.outlier_fixed if c < K], dtype=np.int64)
        fac = np.array([f for c, f in spec.outlier_fixed if c < K], dtype=np.float32)
    else:
        n_out = max(1, int(round(spec.outlier_frac * K)))
        idx = np.sort(rng.choice(K, n_out, replace=False))
        lo, hi = spec.factor_range
        fac = np.exp(rng.uniform(np.log(lo), np.log(hi), n_out)).astype(np.float32)
    X[:, idx] *= fac[None, :]
    w_std = spec.w_std if spec.w_std is not None else 1.0 / np.sqrt(K)
    W = rng.standard_normal((N, K), dtype=np.float32) * np.float32(w_std)
    X_store, Xf = round_to_dtype(X, spec.x_dtype)
    W_store, Wf = round_to_dtype(W, spec.w_dtype)
    del X, W
    chmax = np.abs(Xf).max(axis=0).astype(np.float32)
    T = threshold(spec.t_rule, Xf, chmax, spec.t_value)
    return Layer(spec, X_store, Xf, W_store, Wf, chmax, T, idx)
