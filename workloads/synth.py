"""Seeded synthetic router workloads.

The paper routes tokens of a trained Llama-style MoE (Section 4.1: e in {16, 32, 64}, k = 2,
688 x 512-token batches over 8 GPUs, capacity c = k*n/e from Section 2.3).  Neither its data nor
its router weights exist here, so these generators stand in for them with the same shape class:
softmax-peaked rows and a skewed expert popularity obtained from a per-expert logit bias.

Every array is a pure function of (config name, seed).  bf16 inputs are produced by rounding the
fp32 draw to nearest-even and are returned both as raw 16-bit patterns (what the GPU reads) and
as the exactly equal fp32 values (what a CPU checker widens), so both sides see identical bits.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, Optional

import numpy as np


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round-to-nearest-even; inputs are finite."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounding = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + rounding) >> np.uint32(16)).astype(np.uint16)


def bf16_from_bits(b: np.ndarray) -> np.ndarray:
    """bf16 bit patterns -> the exactly equal fp32 values."""
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_round(a: np.ndarray) -> np.ndarray:
    return bf16_from_bits(bf16_bits(a))


def capacity(T: int, E: int, k: int, factor: float) -> int:
    """c' = c_f * k*n/e (Section 2.3), rounded up."""
    return int(math.ceil(factor * T * k / E - 1e-9))


# name -> shape, dtype, bias recipe.  C is the per-expert capacity; t the SoftTopk temperature.
CONFIGS: Dict[str, dict] = {
    "cfg1": dict(T=64, d=64, E=8, k=2, C=16, dtype="fp32", bias=None, t=0.0),
    "cfg2": dict(T=4096, d=1024, E=16, k=2, C=512, dtype="bf16", bias=("normal", 0.5), t=1.0),
    "cfg3": dict(T=16384, d=2048, E=64, k=8, C=2048, dtype="bf16", bias=("zipf", 1.1), t=1.0),
    "cfg4a": dict(T=32768, d=2048, E=64, k=8, C=5120, dtype="bf16", bias=None, t=1.0),
    "cfg4b_exact": dict(T=32768, d=2048, E=64, k=8, C=5120, dtype="bf16", bias=None, t=1.0,
                        dup=("exact", 0.25)),
    "cfg4b_near": dict(T=32768, d=2048, E=64, k=8, C=5120, dtype="bf16", bias=None, t=1.0,
                       dup=("near", 0.25)),
    "cfg5": dict(T=65536, d=2048, E=128, k=8, C=4096, dtype="bf16", bias=("zipf", 1.2), t=1.0),
}


@dataclasses.dataclass
class RouterInputs:
    name: str
    T: int
    d: int
    E: int
    k: int
    C: int
    t: float
    dtype: str                    # "fp32" or "bf16"
    x: np.ndarray                 # [T, d] fp32 values (bf16-representable when dtype == "bf16")
    W: np.ndarray                 # [d, E] fp32 values (same remark)
    bias: Optional[np.ndarray]    # [E] fp32 or None
    x_bits: Optional[np.ndarray]  # [T, d] uint16 bf16 patterns (dtype == "bf16")
    W_bits: Optional[np.ndarray]  # [d, E] uint16


def _expert_bias(rng: np.random.Generator, E: int, recipe) -> Optional[np.ndarray]:
    if recipe is None:
        return None
    kind, param = recipe
    if kind == "normal":          # N(0, variance = param), i.i.d. per expert
        return (rng.standard_normal(E) * math.sqrt(param)).astype(np.float32)
    if kind == "zipf":            # w_j = j^-s, min-max scaled to [0, 2], expert order shuffled
        w = np.arange(1, E + 1, dtype=np.float64) ** (-param)
        b = 2.0 * (w - w[-1]) / (w[0] - w[-1])
        return rng.permutation(b).astype(np.float32)
    raise ValueError(kind)


def make_inputs(name: str, seed: int = 0, T: Optional[int] = None) -> RouterInputs:
    """Build the (x, W, bias) of a named config.  `T` overrides the token count (capacity keeps
    the config's capacity factor) so that reduced copies of a workload keep its structure."""
    cfg = dict(CONFIGS[name])
    idx = list(CONFIGS).index(name)
    rng = np.random.default_rng([seed, idx])
    d, E, k = cfg["d"], cfg["E"], cfg["k"]
    if T is None:
        T, C = cfg["T"], cfg["C"]
    else:
        factor = cfg["C"] * E / (cfg["T"] * k)
        C = capacity(T, E, k, factor)
    bias = _expert_bias(rng, E, cfg["bias"])
    W = (rng.standard_normal((d, E), dtype=np.float32) * np.float32(1.0 / math.sqrt(d)))
    x = rng.standard_normal((T, d), dtype=np.float32)
    dup = cfg.get("dup")
    if dup is not None:
        kind, frac = dup
        rows = rng.permutation(T)[: int(frac * T)]
        base = x[rows[0]].copy()
        if kind == "exact":
            x[rows] = base
        else:
            x[rows] = base + np.float32(1e-3) * rng.standard_normal((rows.size, d), dtype=np.float32)
    x_bits = W_bits = None
    if cfg["dtype"] == "bf16":
        x_bits, W_bits = bf16_bits(x), bf16_bits(W)
        x, W = bf16_from_bits(x_bits), bf16_from_bits(W_bits)
    return RouterInputs(name=name, T=T, d=d, E=E, k=k, C=C, t=cfg["t"], dtype=cfg["dtype"],
                        x=x, W=W, bias=bias, x_bits=x_bits, W_bits=W_bits)


def make_logits(name: str, seed: int = 0, T: Optional[int] = None, batch: int = 0) -> np.ndarray:
    """fp32 router logits with the distribution x.W + bias has for the named config, drawn
    directly (x ~ N(0,1), W ~ N(0,1/d) give unit-variance logits) so that cases which do not
    exercise the projection need not generate x.  Duplicate-row variants are honoured.
    `batch` > 0 gives another batch of tokens for the SAME router (same seed: same expert bias),
    as successive training steps see it."""
    cfg = dict(CONFIGS[name])
    idx = list(CONFIGS).index(name)
    rng = np.random.default_rng([seed, idx, 7])
    E = cfg["E"]
    T = cfg["T"] if T is None else T
    bias = _expert_bias(rng, E, cfg["bias"])
    if batch > 0:
        rng = np.random.default_rng([seed, idx, 7, batch])
    L = rng.standard_normal((T, E), dtype=np.float32)
    dup = cfg.get("dup")
    if dup is not None:
        kind, frac = dup
        rows = rng.permutation(T)[: int(frac * T)]
        base = L[rows[0]].copy()
        if kind == "exact":
            L[rows] = base
        else:
            L[rows] = base + np.float32(3e-2) * rng.standard_normal((rows.size, E), dtype=np.float32)
    if bias is not None:
        L = L + bias[None, :]
    return np.ascontiguousarray(L, dtype=np.float32)
