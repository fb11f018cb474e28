"""Seeded synthetic inputs for a single DoRA linear module.

This module only draws random numbers and rounds them to the storage dtype.  It
holds none of the method's arithmetic (no factored norm, no compose, no
gradients); the one derived quantity, the magnitude vector, follows the
initialisation the paper describes in Sec. 3.1 (m starts at the row norm of the
frozen weight and stays close to it), which is a property of the *workload*, not
of the method: m = ||W||_row * (1 + jitter).

Both the CPU oracle's tests and the HIP path's tests/bench consume exactly these
arrays, so the two sides see byte-identical, already-quantised inputs.

Storage conventions
-------------------
* dtype "f32": arrays are numpy float32.
* dtype "bf16": arrays are numpy uint16 holding bfloat16 bit patterns
  (round-to-nearest-even from float32).  `to_f64` widens either form exactly.
* dtype "f16": arrays are numpy float16 (IEEE binary16, round-to-nearest-even,
  overflow to infinity beyond 65504).
* m is always float32.  s is a float32 scalar (rsLoRA: alpha / sqrt(r)).
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict

import numpy as np

BASE_SEED = 260322276
TENSOR_IDS = {"W": 0, "A": 1, "B": 2, "m": 3, "x": 4, "dy": 5, "mask": 6}


@dataclass(frozen=True)
class DoraConfig:
    """Shape and value-distribution recipe of one module."""

    name: str
    d_out: int
    d_in: int
    r: int
    tokens: int
    dtype: str  # "f32" | "bf16" | "f16"
    alpha: float  # s = alpha / sqrt(r)
    sigma_B: float  # std of B entries
    sigma_m: float = 1e-3  # std of the relative jitter on m
    seed_offset: int = 0

    @property
    def s(self) -> np.float32:
        return np.float32(self.alpha / np.sqrt(float(self.r)))

    @property
    def eps(self) -> float:
        # dtype-aware epsilon of the forward contract (App. A item 2)
        return 1e-12 if self.dtype == "f32" else 1e-6

    def scaled(self, **kw) -> "DoraConfig":
        return replace(self, **kw)


# The five workload families.  Value distributions: W, A ~ N(0, var 1/d_in);
# B ~ N(0, std sigma_B); x, dy ~ N(0, 1); m = ||W||_row (1 + N(0, std 1e-3)).
C1 = DoraConfig("C1_f32_256x512_r16", 256, 512, 16, 64, "f32", 16.0, 1e-2, seed_offset=1000)
C2 = DoraConfig("C2_bf16_4096x4096_r384", 4096, 4096, 384, 4096, "bf16", 32.0, 1e-3, seed_offset=2000)
C3 = DoraConfig("C3_bf16_8192x8192_r384", 8192, 8192, 384, 8192, "bf16", 32.0, 1e-3, seed_offset=3000)
C4_UP = DoraConfig("C4_bf16_up_27648x5120_r384", 27648, 5120, 384, 8192, "bf16", 32.0, 1e-3, seed_offset=4000)
C4_DOWN = DoraConfig("C4_bf16_down_5120x27648_r384", 5120, 27648, 384, 8192, "bf16", 32.0, 1e-3, seed_offset=4100)

# 8B-class decoder layer: hidden 4096, 32 heads x 128, 8 KV heads, intermediate 14336.
C5_MODULE_SHAPES = (
    ("q", 4096, 4096),
    ("k", 1024, 4096),
    ("v", 1024, 4096),
    ("o", 4096, 4096),
    ("gate", 14336, 4096),
    ("up", 14336, 4096),
    ("down", 4096, 14336),
)


def c5_module(module_index: int, r: int, layer: int = 0, tokens: int = 4096) -> DoraConfig:
    name, d_out, d_in = C5_MODULE_SHAPES[module_index]
    return DoraConfig(
        f"C5_bf16_L{layer}_{name}_{d_out}x{d_in}_r{r}", d_out, d_in, r, tokens, "bf16", 32.0, 1e-3,
        seed_offset=5000 + 100 * layer + 10 * module_index + 100000 * r,
    )


def stress(cfg: DoraConfig) -> DoraConfig:
    """Variant in which all three terms of the squared norm are O(1).

    With the stock sigma_B the low-rank terms move the norm by less than the
    bf16 tolerance, so a kernel that dropped them would still pass; raising
    sigma_B until s^2 r sigma_B^2 ~ 1 closes that hole.
    """
    sigma = 1.0 / (float(cfg.s) * np.sqrt(float(cfg.r)))
    return replace(cfg, name=cfg.name + "_stressB", sigma_B=float(sigma), seed_offset=cfg.seed_offset + 500)


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32)
    nan = np.isnan(a)
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    rounded = (bits + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    out = rounded.astype(np.uint16)
    if nan.any():
        out[nan] = np.uint16(0x7FC0)
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def quantise(a64: np.ndarray, dtype: str) -> np.ndarray:
    """One rounding from the generator's float64/float32 values to the storage dtype."""
    if dtype == "f32":
        return np.ascontiguousarray(a64, dtype=np.float32)
    if dtype == "bf16":
        return f32_to_bf16_bits(np.asarray(a64, dtype=np.float32))
    if dtype == "f16":
        with np.errstate(over="ignore"):
            return np.ascontiguousarray(np.asarray(a64, dtype=np.float32).astype(np.float16))
    raise ValueError(f"unknown dtype {dtype!r}")


def to_f64(a: np.ndarray) -> np.ndarray:
    """Exact widening of a stored array (float32, or uint16 bf16 bits) to float64."""
    if a.dtype == np.uint16:
        return bf16_bits_to_f32(a).astype(np.float64)
    return np.asarray(a, dtype=np.float64)


def _normal(seed: int, shape, std: float) -> np.ndarray:
    rng = np.random.Generator(np.random.Philox(seed))
    out = rng.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        out *= np.float32(std)
    return out


def dropped_input(cfg: DoraConfig, x: np.ndarray, p: float) -> np.ndarray:
    """The adapter branch's input under LoRA dropout with probability p: x (.) keep / (1 - p), keep drawn
    from the tensor's own Philox stream, rounded once to the storage dtype.  Dropout itself is outside the
    module: its random numbers reach both the oracle and the HIP path as this input."""
    rng = np.random.Generator(np.random.Philox(BASE_SEED + cfg.seed_offset + TENSOR_IDS["mask"]))
    keep = rng.random(size=x.shape, dtype=np.float32) >= np.float32(p)
    return quantise(to_f64(x) * keep / (1.0 - p), cfg.dtype)


def make_inputs(cfg: DoraConfig, with_dy: bool = True) -> Dict[str, np.ndarray]:
    """Draw W, A, B, m, x (and dy) for `cfg`.

    Returns the *stored* arrays (see module docstring) plus "s" (float32) and
    "eps" (float).  Every tensor has its own Philox stream:
    seed = BASE_SEED + cfg.seed_offset + tensor_id.
    """
    base = BASE_SEED + cfg.seed_offset
    inv = 1.0 / np.sqrt(float(cfg.d_in))
    W = quantise(_normal(base + TENSOR_IDS["W"], (cfg.d_out, cfg.d_in), inv), cfg.dtype)
    A = quantise(_normal(base + TENSOR_IDS["A"], (cfg.r, cfg.d_in), inv), cfg.dtype)
    B = quantise(_normal(base + TENSOR_IDS["B"], (cfg.d_out, cfg.r), cfg.sigma_B), cfg.dtype)
    x = quantise(_normal(base + TENSOR_IDS["x"], (cfg.tokens, cfg.d_in), 1.0), cfg.dtype)
    # magnitude: row norm of the stored (already rounded) W, times a near-unity jitter
    W64 = to_f64(W)
    row_norm = np.sqrt(np.einsum("ij,ij->i", W64, W64))
    del W64
    jitter = _normal(base + TENSOR_IDS["m"], (cfg.d_out,), cfg.sigma_m).astype(np.float64)
    m = (row_norm * (1.0 + jitter)).astype(np.float32)
    out = {"W": W, "A": A, "B": B, "m": m, "x": x, "s": cfg.s, "eps": cfg.eps}
    if with_dy:
        out["dy"] = quantise(_normal(base + TENSOR_IDS["dy"], (cfg.tokens, cfg.d_out), 1.0), cfg.dtype)
    return out
