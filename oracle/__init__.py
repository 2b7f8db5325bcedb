"""Python face of the CPU oracle (oracle/atb_oracle.c) -- test infrastructure.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package.  It holds the plain definition of BFP16 quantise / decode and of
the fp64-accumulated GEMM of arXiv 2511.16041's BFP16 x BF16 path, plus
(oracle.model) the paper's analytical model.  Nothing here touches the GPU
library, and the GPU library never falls back to it.
"""
from __future__ import annotations

import ctypes
from typing import Optional, Sequence, Tuple

import numpy as np

from . import build as _build
from . import model  # noqa: F401  (re-exported)

_lib = None


def _load():
    global _lib
    if _lib is not None:
        return _lib
    lib = ctypes.CDLL(_build.ensure_built())
    i64, p = ctypes.c_int64, ctypes.c_void_p
    lib.atb_oracle_bf16_to_double.restype = ctypes.c_double
    lib.atb_oracle_bf16_to_double.argtypes = [ctypes.c_uint16]
    lib.atb_oracle_bf16_from_double.restype = ctypes.c_uint16
    lib.atb_oracle_bf16_from_double.argtypes = [ctypes.c_double]
    lib.atb_oracle_bf16_from_double_array.restype = None
    lib.atb_oracle_bf16_from_double_array.argtypes = [p, i64, p]
    lib.atb_oracle_bfp16_quantize.restype = i64
    lib.atb_oracle_bfp16_quantize.argtypes = [p, i64, i64, i64, p, p]
    lib.atb_oracle_bfp16_decode.restype = ctypes.c_int
    lib.atb_oracle_bfp16_decode.argtypes = [p, p, i64, i64, p]
    lib.atb_oracle_gemm_rows.restype = ctypes.c_int
    lib.atb_oracle_gemm_rows.argtypes = [p, p, p, i64, i64, i64, p, i64, p, p, p]
    lib.atb_oracle_gemm_tiled.restype = ctypes.c_int
    lib.atb_oracle_gemm_tiled.argtypes = [p, p, p, i64, i64, i64,
                                          ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, p, p]
    _lib = lib
    return lib


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def bf16_to_double(bits) -> np.ndarray:
    """bf16 bit patterns (uint16) -> float64, exactly."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def bf16_from_double_scalar(x: float) -> int:
    return int(_load().atb_oracle_bf16_from_double(float(x)))


def bf16_from_double(x) -> np.ndarray:
    """float64 -> bf16 bit patterns, one RNE rounding (element loop in C)."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    out = np.empty(x.shape, dtype=np.uint16)
    _load().atb_oracle_bf16_from_double_array(_ptr(x), x.size, _ptr(out))
    return out


def quantize(A: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """fp32 A[M][K] -> (mant int8[M][K], expo uint8[M][K/8])."""
    A = np.ascontiguousarray(A, dtype=np.float32)
    M, K = A.shape
    mant = np.empty((M, K), dtype=np.int8)
    expo = np.empty((M, K // 8), dtype=np.uint8)
    rc = _load().atb_oracle_bfp16_quantize(_ptr(A), M, K, K, _ptr(mant), _ptr(expo))
    if rc != 0:
        raise ValueError(f"atb_oracle_bfp16_quantize returned {rc} (bad argument or non-finite input)")
    return mant, expo


def decode(mant: np.ndarray, expo: np.ndarray) -> np.ndarray:
    mant = np.ascontiguousarray(mant, dtype=np.int8)
    expo = np.ascontiguousarray(expo, dtype=np.uint8)
    M, K = mant.shape
    out = np.empty((M, K), dtype=np.float64)
    rc = _load().atb_oracle_bfp16_decode(_ptr(mant), _ptr(expo), M, K, _ptr(out))
    if rc != 0:
        raise ValueError("atb_oracle_bfp16_decode: bad argument")
    return out


def gemm(mant: np.ndarray, expo: np.ndarray, B_bits: np.ndarray,
         rows: Optional[Sequence[int]] = None, want_sum: bool = False):
    """C_ref (bf16 bits), T = sum |a||b| (fp64) [, S = fp64 sum before rounding]
    for all rows, or for the listed rows only.  Also returns the thread count."""
    mant = np.ascontiguousarray(mant, dtype=np.int8)
    expo = np.ascontiguousarray(expo, dtype=np.uint8)
    B_bits = np.ascontiguousarray(B_bits, dtype=np.uint16)
    M, K = mant.shape
    K2, N = B_bits.shape
    assert K2 == K and expo.shape == (M, K // 8)
    if rows is None:
        rows_arr, nrows = None, M
    else:
        rows_arr = np.ascontiguousarray(rows, dtype=np.int64)
        nrows = rows_arr.size
    C = np.empty((nrows, N), dtype=np.uint16)
    T = np.empty((nrows, N), dtype=np.float64)
    S = np.empty((nrows, N), dtype=np.float64) if want_sum else None
    th = _load().atb_oracle_gemm_rows(_ptr(mant), _ptr(expo), _ptr(B_bits), M, N, K,
                                      _ptr(rows_arr), nrows, _ptr(C), _ptr(S), _ptr(T))
    if th < 0:
        raise ValueError("atb_oracle_gemm_rows: bad argument")
    if want_sum:
        return C, T, S, th
    return C, T, th


def gemm_tiled(mant, expo, B_bits, T_MA: int, T_MC: int, T_K: int, T_N: int):
    """The ATB loop nest of the paper, written out; returns (C bits, switches)."""
    mant = np.ascontiguousarray(mant, dtype=np.int8)
    expo = np.ascontiguousarray(expo, dtype=np.uint8)
    B_bits = np.ascontiguousarray(B_bits, dtype=np.uint16)
    M, K = mant.shape
    N = B_bits.shape[1]
    C = np.zeros((M, N), dtype=np.uint16)
    sw = ctypes.c_int64(0)
    rc = _load().atb_oracle_gemm_tiled(_ptr(mant), _ptr(expo), _ptr(B_bits), M, N, K,
                                       T_MA, T_MC, T_K, T_N, _ptr(C), ctypes.byref(sw))
    if rc != 0:
        raise ValueError("atb_oracle_gemm_tiled: bad argument")
    return C, int(sw.value)


def bfp16_as_bf16_bits(mant: np.ndarray, expo: np.ndarray) -> np.ndarray:
    """BFP16 values as bf16 bit patterns.  Exact: m * 2^(E-133) with |m| <= 127 has at most 7
    significant bits (Sec. 2.4), bf16 keeps 8; asserted rather than assumed."""
    v = decode(mant, expo)
    bits = bf16_from_double(v)
    assert np.array_equal(bf16_to_double(bits), v), "a BFP16 value outside the bf16 range"
    return bits


def tolerance(T: np.ndarray) -> np.ndarray:
    """Acceptance bound per element: 2^-7 * sum_k |a||b| + 1e-6."""
    return T * 2.0 ** -7 + 1e-6
