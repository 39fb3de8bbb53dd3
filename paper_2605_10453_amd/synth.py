"""Seeded synthetic inputs for the drafter LM-head (hidden states and head weights).

This module only draws random numbers, scales them and rounds them to bf16.  It
holds none of the head's arithmetic (no projection, no softmax, no top-k), so the
HIP path and the CPU checker can both be fed from it without sharing any of the
method's code.  Everything is numpy on the host; bf16 values travel as uint16
bit patterns.

Shapes follow the drafter head of the paper's section 4.1 in row-vector form:
h is [rows, d], A (the transposed down-projection) is [d, r], B (the transposed
up-projection) is [r, V], W (the transposed full head) is [d, V].
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np


# --------------------------------------------------------------------------- bf16

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even), returned as uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    # NaN stays NaN (quiet); everything else: add 0x7fff + lsb, then truncate.
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    rounded = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    nan = np.isnan(x)
    out = rounded.astype(np.uint16)
    if nan.any():
        out = np.where(nan, np.uint16(0x7FC0), out)
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to fp32 exactly."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to fp64 exactly."""
    return bf16_bits_to_f32(b).astype(np.float64)


# --------------------------------------------------------------------------- configs

@dataclass(frozen=True)
class HeadConfig:
    name: str
    rows: int
    d: int
    r: int
    V: int
    k: int
    peaked_every: int = 0   # rows with i % peaked_every == 0 are scaled by 4 (0 = none)


# The five workloads: a tiny case, two single-row latency shapes, the 512-row
# throughput shape and the large-target shape.
CONFIGS = {
    "C1": HeadConfig("C1", rows=1, d=256, r=32, V=8192, k=8),
    "C2": HeadConfig("C2", rows=1, d=4096, r=512, V=128256, k=10),
    "C3": HeadConfig("C3", rows=1, d=5120, r=640, V=151936, k=10),
    "C4": HeadConfig("C4", rows=512, d=4096, r=512, V=128256, k=10, peaked_every=10),
    "C4_r256": HeadConfig("C4_r256", rows=512, d=4096, r=256, V=128256, k=10, peaked_every=10),
    "C4_r1024": HeadConfig("C4_r1024", rows=512, d=4096, r=1024, V=128256, k=10, peaked_every=10),
    "C5": HeadConfig("C5", rows=256, d=8192, r=1024, V=128256, k=16),
}


@dataclass
class HeadInputs:
    cfg: HeadConfig
    seed: int
    h: np.ndarray                  # uint16 [rows, d]   bf16 bits
    A: np.ndarray                  # uint16 [d, r]      bf16 bits
    B: np.ndarray                  # uint16 [r, V]      bf16 bits
    W: Optional[np.ndarray] = None  # uint16 [d, V]     bf16 bits (independent full head)


def _normal_bf16(rng: np.random.Generator, shape, scale: float, block_rows: int = 256) -> np.ndarray:
    """N(0, scale^2) draws rounded to bf16, generated in row blocks to bound memory."""
    out = np.empty(shape, dtype=np.uint16)
    n0 = shape[0]
    for s in range(0, n0, block_rows):
        e = min(n0, s + block_rows)
        blk = rng.standard_normal((e - s,) + tuple(shape[1:]), dtype=np.float32)
        if scale != 1.0:
            blk *= np.float32(scale)
        out[s:e] = f32_to_bf16_bits(blk)
    return out


def make_inputs(cfg: HeadConfig, seed: int = 0, with_full_head: bool = False) -> HeadInputs:
    """Draw (h, A, B[, W]) for one workload.

    Draw order is h, A, B, W from one numpy Generator(seed).  h ~ N(0,1);
    A and W have variance 1/d, B has variance 1/r, so that both t = h*A and the
    logits have unit variance per row.  Values are rounded once to bf16.
    Rows i with i % peaked_every == 0 are multiplied by 4 (exact in bf16) to give
    some rows a much sharper softmax.
    """
    rng = np.random.default_rng(seed)
    h = _normal_bf16(rng, (cfg.rows, cfg.d), 1.0)
    A = _normal_bf16(rng, (cfg.d, cfg.r), cfg.d ** -0.5)
    B = _normal_bf16(rng, (cfg.r, cfg.V), cfg.r ** -0.5)
    W = _normal_bf16(rng, (cfg.d, cfg.V), cfg.d ** -0.5) if with_full_head else None
    if cfg.peaked_every:
        hf = bf16_bits_to_f32(h)
        hf[:: cfg.peaked_every] *= np.float32(4.0)
        h = f32_to_bf16_bits(hf)
    return HeadInputs(cfg=cfg, seed=seed, h=h, A=A, B=B, W=W)


def small_config(rows: int, d: int, r: int, V: int, k: int, peaked_every: int = 0,
                 name: str = "custom") -> HeadConfig:
    return HeadConfig(name, rows=rows, d=d, r=r, V=V, k=k, peaked_every=peaked_every)


# --------------------------------------------------------------------------- planted ties

def plant_identical_columns(M: np.ndarray, column_values_f64: np.ndarray, ids) -> np.ndarray:
    """Overwrite columns `ids` of the bf16 matrix M ([K, V] bits) with one common column.

    `column_values_f64` ([K]) is rounded once to bf16 and the same bit pattern is
    written to every listed column, so any head evaluated on M sees bit-identical
    weights at those vocabulary ids (hence exactly tied logits).  The caller
    chooses the values; nothing is computed here beyond the rounding.
    """
    col = f32_to_bf16_bits(np.asarray(column_values_f64, dtype=np.float64).astype(np.float32))
    for v in ids:
        M[:, int(v)] = col
    return M
