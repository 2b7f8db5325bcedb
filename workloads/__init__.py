"""Seeded synthetic inputs for the BFP16 x BF16 GEMM workloads.

This module only draws random numbers and casts them to the storage types of
the inputs (fp32 for the un-quantised A, bf16 bit patterns for B).  It holds
none of the method's arithmetic (no BFP16 quantisation, no decode, no GEMM) so
that both the CPU oracle's tests and the GPU library's tests / bench can use
it without sharing code with each other.

Recipe (numpy.random.default_rng(seed), draws in this order):
  1. A0  = standard normals, M x K, fp32, row-major
  2. u_i = integers uniform in [-row_exp, +row_exp], one per row; A = A0 * 2^u_i
  3. (config "ragged") outlier mask: each element independently with p = 0.01
     is multiplied by 2^8
  4. B   = normals (sigma given) or uniform(-1, 1), K x N, fp32, rounded to
     bf16 with round-to-nearest-even
The paper measures on synthetic GEMM shapes only (its Tables 2 and 3), so
these stand in for nothing else.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Tuple

import numpy as np


@dataclass(frozen=True)
class GemmConfig:
    name: str
    M: int
    N: int
    K: int
    row_exp: int            # rows of A scaled by 2^U{-row_exp..row_exp}
    b_dist: str             # "normal" or "uniform"
    b_sigma: float          # sigma for "normal"
    outlier_p: float        # probability of a x2^8 outlier in A
    seed: int = 0


# The five workloads (shapes and distributions only; tile factors are chosen
# by the caller).
CONFIGS: Dict[str, GemmConfig] = {
    "small256": GemmConfig("small256", 256, 256, 256, 4, "normal", 1.0, 0.0),
    "square4096": GemmConfig("square4096", 4096, 4096, 4096, 4, "normal", 1.0, 0.0),
    "square8192": GemmConfig("square8192", 8192, 8192, 8192, 4, "normal", 1.0, 0.0),
    "mlp": GemmConfig("mlp", 8192, 14336, 4096, 6, "normal", 0.02, 0.0),
    "ragged": GemmConfig("ragged", 3000, 5000, 4104, 4, "uniform", 1.0, 0.01),
}


def fp32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Storage cast fp32 -> bf16 bit patterns (uint16), round to nearest even.
    Finite inputs only."""
    w = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (w >> np.uint32(16)) & np.uint32(1)
    return ((w + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_fp32(bits: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def make_inputs(cfg: GemmConfig, M: int | None = None, N: int | None = None,
                K: int | None = None) -> Tuple[np.ndarray, np.ndarray]:
    """Returns (A fp32 [M][K], B bf16 bits uint16 [K][N]).  M, N, K override the
    config's shape (same distributions) for reduced-size test cases."""
    M = cfg.M if M is None else M
    N = cfg.N if N is None else N
    K = cfg.K if K is None else K
    rng = np.random.default_rng(cfg.seed)
    A = rng.standard_normal((M, K), dtype=np.float32)
    u = rng.integers(-cfg.row_exp, cfg.row_exp + 1, size=M)
    A *= np.exp2(u).astype(np.float32)[:, None]
    if cfg.outlier_p > 0.0:
        mask = rng.random((M, K), dtype=np.float32) < np.float32(cfg.outlier_p)
        A[mask] *= np.float32(256.0)
    if cfg.b_dist == "normal":
        Bf = rng.standard_normal((K, N), dtype=np.float32)
        if cfg.b_sigma != 1.0:
            Bf *= np.float32(cfg.b_sigma)
    elif cfg.b_dist == "uniform":
        Bf = rng.random((K, N), dtype=np.float32) * np.float32(2.0) - np.float32(1.0)
    else:
        raise ValueError(cfg.b_dist)
    return A, fp32_to_bf16_bits(Bf)


def small_integer_inputs(M: int, N: int, K: int, seed: int = 0,
                         amax: int = 4, bmax: int = 4) -> Tuple[np.ndarray, np.ndarray]:
    """Inputs whose products and sums are small integers (|sum| < 2^24), so any
    summation order in fp32 is exact.  A values are integers in [-amax, amax]
    times a per-row power of two; B integers in [-bmax, bmax]."""
    rng = np.random.default_rng(seed)
    A = rng.integers(-amax, amax + 1, size=(M, K)).astype(np.float32)
    u = rng.integers(-3, 4, size=M)
    A *= np.exp2(u).astype(np.float32)[:, None]
    Bf = rng.integers(-bmax, bmax + 1, size=(K, N)).astype(np.float32)
    return A, fp32_to_bf16_bits(Bf)
