"""Seeded synthetic inputs for the RSR matvec workloads.

This module is the only code shared by the CPU oracle's tests and the HIP
path's tests/benchmark.  It draws matrices and vectors and nothing else: none
of the method's arithmetic (no encoding, sorting, packing or multiplying)
lives here.  All draws use numpy's PCG64 with an explicit seed, so every test
and benchmark input can be regenerated exactly.

The five workload families mirror the shapes and value distributions the
paper's experiments imply (binary matrix x float32 vector micro-benchmarks;
ternary LLM layer shapes; a retrieval/ranking table); they stand in for the
paper's trained models and datasets, which are not available offline.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Tuple

import numpy as np

BASE_SEED = 0x525352  # "RSR"


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


# ----------------------------------------------------------------- matrices
def binary_matrix(rows: int, cols: int, p_one: float = 0.5, seed: int = BASE_SEED) -> np.ndarray:
    """Entries i.i.d. Bernoulli(p_one) in {0,1}, int8 row-major."""
    return (_rng(seed).random((rows, cols), dtype=np.float32) < p_one).astype(np.int8)


def ternary_matrix(rows: int, cols: int, p_zero: float = 1.0 / 3.0,
                   seed: int = BASE_SEED) -> np.ndarray:
    """Entries i.i.d. with P(0)=p_zero and P(+1)=P(-1)=(1-p_zero)/2, int8."""
    u = _rng(seed).random((rows, cols), dtype=np.float32)
    half = (1.0 - p_zero) / 2.0
    M = np.zeros((rows, cols), dtype=np.int8)
    M[u < half] = 1
    M[(u >= half) & (u < 2.0 * half)] = -1
    return M


def column_density_binary(rows: int, cols: int, lo: float = 0.05, hi: float = 0.5,
                          seed: int = BASE_SEED, chunk_rows: int = 1 << 16) -> np.ndarray:
    """Binary table whose column j has its own density p_j ~ U[lo, hi]."""
    g = _rng(seed)
    p = g.uniform(lo, hi, size=cols).astype(np.float32)
    M = np.empty((rows, cols), dtype=np.int8)
    for r0 in range(0, rows, chunk_rows):
        r1 = min(rows, r0 + chunk_rows)
        M[r0:r1] = g.random((r1 - r0, cols), dtype=np.float32) < p[None, :]
    return M


def dictionary_binary_matrix(rows: int, cols: int, k: int, patterns: int,
                             seed: int = BASE_SEED) -> np.ndarray:
    """Binary matrix whose columns, inside every block of k rows, are drawn from a
    dictionary of `patterns` random k-entry patterns (heavy redundancy: few groups, long)."""
    g = _rng(seed)
    M = np.zeros((rows, cols), dtype=np.int8)
    for r0 in range(0, rows, k):
        r1 = min(rows, r0 + k)
        words = (g.random((k, patterns), dtype=np.float32) < 0.5).astype(np.int8)
        pick = g.integers(0, patterns, size=cols)
        M[r0:r1] = words[: r1 - r0, pick]
    return M


# ------------------------------------------------------------------ vectors
def normal_f32(n: int, seed: int = BASE_SEED + 1) -> np.ndarray:
    return _rng(seed).standard_normal(n, dtype=np.float32)


def uniform_f32(n: int, seed: int = BASE_SEED + 1) -> np.ndarray:
    return _rng(seed).random(n, dtype=np.float32)


def integer_f32(n: int, lo: int = -8, hi: int = 8, seed: int = BASE_SEED + 2) -> np.ndarray:
    """Integer-valued vector (uniform ints in [lo, hi]) stored as float32."""
    return _rng(seed).integers(lo, hi + 1, size=n).astype(np.float32)


def to_bf16(x: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Round float32 samples to bfloat16 (round-to-nearest-even).

    Returns (bits uint16, values float32): the bf16 storage the GPU receives
    and the same numbers widened back, which is what the oracle multiplies.
    """
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    rounded = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    bits = rounded.astype(np.uint16)
    vals = (bits.astype(np.uint32) << 16).view(np.float32)
    return bits, vals


def normal_bf16(n: int, seed: int = BASE_SEED + 1):
    return to_bf16(normal_f32(n, seed))


# ----------------------------------------------------------------- workloads
@dataclass(frozen=True)
class Layer:
    name: str
    rows: int     # outputs
    cols: int     # inputs (length of v)


# 2B-class ternary LLM: hidden 2560, kv 640, ffn 6912.
LLM_2B_LAYERS: List[Layer] = [
    Layer("q", 2560, 2560), Layer("k", 640, 2560), Layer("v", 640, 2560),
    Layer("o", 2560, 2560), Layer("gate", 6912, 2560), Layer("up", 6912, 2560),
    Layer("down", 2560, 6912),
]
LLM_2B_P_ZERO = 0.4

# 8B-class ternary LLM: hidden 4096, ffn 14336.
LLM_8B_LAYERS: List[Layer] = [
    Layer("up", 14336, 4096), Layer("down", 4096, 14336), Layer("attn", 4096, 4096),
]
LLM_8B_P_ZERO = 0.35

# The shape the headline metric is quoted on (an 8B-class down projection).
METRIC_LAYER = Layer("down", 4096, 14336)


def metric_matrix(seed: int = BASE_SEED + 40) -> np.ndarray:
    return ternary_matrix(METRIC_LAYER.rows, METRIC_LAYER.cols, LLM_8B_P_ZERO, seed)
