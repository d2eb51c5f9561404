"""Seeded synthetic inputs shaped like the paper's workloads.

This module serves both the HIP path and the CPU oracle's tests, so it holds
none of the method's arithmetic: only shapes, seeds, random draws and the
bf16 storage rounding of the inputs.  It imports numpy only.

Shapes: ImageNet 256x256 with a stride-16 tokenizer gives a 16x16 token grid
(N = 256, Section 4.1 "Training Details"); the 384x384 setting gives 24x24
(N = 576, Table 3); model widths / head counts are Table 1 (head dim 64
everywhere).  The trained activations and the data set are not available, so
q, k, v are Gaussians of standard deviation 1/sqrt(d) and the per-head base
decay is uniform in a stated range.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    B: int            # batch
    Hh: int           # heads
    d: int            # head dim (dk = dv)
    grid_h: int
    grid_w: int
    dtype: str        # "f32" or "bf16": storage type of q, k, v
    gamma_lo: float
    gamma_hi: float
    seed: int
    kind: str = "prefill"   # "prefill" or "decode"
    steps: int = 0          # decode only: consecutive raster positions walked

    @property
    def N(self) -> int:
        return self.grid_h * self.grid_w


# The five benchmark / parity configurations.
TINY = Workload("tiny_oracle", 1, 1, 32, 8, 8, "f32", 0.90, 0.99, 1001)
BASE_PREFILL = Workload("base_prefill_16x16", 8, 12, 64, 16, 16, "bf16", 0.85, 0.999, 1002)
LARGE_PREFILL = Workload("large_prefill_24x24", 32, 16, 64, 24, 24, "bf16", 0.85, 0.999, 1003)
AR_DECODE = Workload("ar_decode_16x16", 256, 20, 64, 16, 16, "bf16", 0.85, 0.999, 1004,
                     kind="decode", steps=256)
HIGHRES = Workload("highres_64x64", 4, 24, 64, 64, 64, "bf16", 0.90, 0.9999, 1005)

CONFIGS = {w.name: w for w in (TINY, BASE_PREFILL, LARGE_PREFILL, AR_DECODE, HIGHRES)}


def scaled(w: Workload, **kw) -> Workload:
    """A copy of a workload with some fields replaced (smaller batch, other grid...)."""
    return replace(w, **kw)


# ---- bf16 storage format (1 sign, 8 exponent, 7 mantissa bits) -------------

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16, round-to-nearest-even; returns the uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    rounding = ((u >> 16) & 1) + np.uint32(0x7FFF)
    out = ((u + rounding) >> 16).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        out[nan] = 0x7FC0
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def store_round(x: np.ndarray, dtype: str) -> np.ndarray:
    """The float32 values that survive storage in `dtype` ("f32" keeps them, "bf16" rounds RNE)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "f32":
        return x
    if dtype == "bf16":
        return bf16_bits_to_f32(f32_to_bf16_bits(x))
    raise ValueError(dtype)


# ---- generators ---------------------------------------------------------------

def gammas(w: Workload, rng: np.random.Generator) -> np.ndarray:
    return rng.uniform(w.gamma_lo, w.gamma_hi, size=(w.Hh,)).astype(np.float32)


def prefill_inputs(w: Workload, layout: str = "bnhd"):
    """q, k, v float32 arrays holding storage-rounded values, plus gamma[Hh] float32.

    layout "bnhd": shape [B, N, Hh, d] (token-major, the primary layout);
    layout "bhnd": the same values returned as a [B, Hh, N, d]-contiguous array
    transposed back to the logical [B, N, Hh, d] view (a strided view).
    Draw order: q, k, v (standard normal, scaled by 1/sqrt(d)), then gamma.
    """
    rng = np.random.default_rng(w.seed)
    shape = (w.B, w.N, w.Hh, w.d)
    scale = np.float32(1.0 / np.sqrt(w.d))
    out = []
    for _ in range(3):
        x = rng.standard_normal(size=shape, dtype=np.float32) * scale
        x = store_round(x, w.dtype)
        if layout == "bhnd":
            x = np.ascontiguousarray(x.transpose(0, 2, 1, 3)).transpose(0, 2, 1, 3)
        elif layout != "bnhd":
            raise ValueError(layout)
        out.append(x)
    g = gammas(w, rng)
    return out[0], out[1], out[2], g


def decode_inputs(w: Workload, steps: int | None = None):
    """q, k, v of shape [steps, B, Hh, d] (one token per step for every sequence) and gamma[Hh]."""
    steps = w.steps if steps is None else steps
    rng = np.random.default_rng(w.seed)
    shape = (steps, w.B, w.Hh, w.d)
    scale = np.float32(1.0 / np.sqrt(w.d))
    out = []
    for _ in range(3):
        x = rng.standard_normal(size=shape, dtype=np.float32) * scale
        out.append(store_round(x, w.dtype))
    g = gammas(w, rng)
    return out[0], out[1], out[2], g


def random_state(w: Workload, seed: int) -> np.ndarray:
    """A float32 carried state [B, Hh, d, d] for carried-state tests."""
    rng = np.random.default_rng(seed)
    return rng.standard_normal(size=(w.B, w.Hh, w.d, w.d), dtype=np.float32) * np.float32(0.5)


def gate_inputs(shape, dtype: str, seed: int) -> np.ndarray:
    """A synthetic post-sigmoid gate lambda in (0, 1) of the given shape: sigmoid of N(2, 1) draws
    (median 0.88, a long tail towards small values), rounded to the storage type.  Stands in for
    the trained gate sigmoid(Linear(x)) of Algorithm 1, which is not available."""
    rng = np.random.default_rng(seed)
    z = rng.standard_normal(size=shape, dtype=np.float32) + np.float32(2.0)
    lam = (1.0 / (1.0 + np.exp(-z.astype(np.float64)))).astype(np.float32)
    lam = store_round(lam, dtype)
    return np.minimum(lam, np.float32(1.0))
