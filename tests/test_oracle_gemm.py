"""Pins for the oracle's GEMM (CPU only): exact rational brute force on tiny
cases, structured matrices with known products, exact-arithmetic inputs, a
library fp64 matmul, and invariance under the ATB loop nest."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
import workloads


def _frac_bf16(bits: int) -> Fraction:
    s = -1 if bits & 0x8000 else 1
    E, f = (bits >> 7) & 0xFF, bits & 0x7F
    if E == 0:
        return s * Fraction(f, 128) * Fraction(2) ** -126
    return s * (1 + Fraction(f, 128)) * Fraction(2) ** (E - 127)


def _round_frac_to_bf16(x: Fraction) -> int:
    """RNE of an exact rational to bf16 via exact integer arithmetic (normal range)."""
    if x == 0:
        return 0
    sign = 0x8000 if x < 0 else 0
    ax = abs(x)
    e = 0
    while Fraction(2) ** (e + 1) <= ax:
        e += 1
    while Fraction(2) ** e > ax:
        e -= 1
    y = ax / Fraction(2) ** (e - 7)              # in [128, 256)
    fl = y.numerator // y.denominator
    fr = y - fl
    r = fl + (1 if fr > Fraction(1, 2) or (fr == Fraction(1, 2) and fl % 2 == 1) else 0)
    if r == 256:
        r, e = 128, e + 1
    assert -126 <= e <= 127
    return sign | ((e + 127) << 7) | (r - 128)


@pytest.mark.parametrize("M,N,K,seed", [(1, 1, 8, 0), (3, 4, 8, 1), (4, 3, 16, 2), (2, 5, 24, 3)])
def test_gemm_tiny_vs_exact_rationals(M, N, K, seed):
    rng = np.random.default_rng(seed)
    A = (rng.standard_normal((M, K)) * np.exp2(rng.integers(-4, 5, size=(M, 1)))).astype(np.float32)
    Bb = workloads.fp32_to_bf16_bits(rng.standard_normal((K, N)).astype(np.float32))
    mant, expo = oracle.quantize(A)
    C, T, S, _ = oracle.gemm(mant, expo, Bb, want_sum=True)
    for i in range(M):
        for j in range(N):
            acc, tacc = Fraction(0), Fraction(0)
            for k in range(K):
                a = Fraction(int(mant[i, k])) * Fraction(2) ** (int(expo[i, k // 8]) - 133)
                b = _frac_bf16(int(Bb[k, j]))
                acc += a * b
                tacc += abs(a) * abs(b)
            # the fp64 sum is within K ulps of the exact sum; the bf16 result equals the RNE of the
            # exact sum unless that sum sits within the fp64 error of a rounding boundary (not for these seeds)
            assert abs(Fraction(float(S[i, j])) - acc) <= Fraction(K, 2 ** 50) * tacc
            assert abs(Fraction(float(T[i, j])) - tacc) <= Fraction(K, 2 ** 50) * tacc
            assert int(C[i, j]) == _round_frac_to_bf16(acc)


def test_gemm_transposed_operands_would_fail():
    """A deliberately asymmetric case with a known answer: A = e_0 e_1^T scaled,
    B has a single non-zero row.  C[0][j] = a * B[1][j]; a row/column mix-up
    anywhere gives zeros instead."""
    M, N, K = 3, 5, 8
    A = np.zeros((M, K), np.float32)
    A[0, 1] = 2.0
    Bf = np.zeros((K, N), np.float32)
    Bf[1] = [1, 2, 3, 4, 5]
    Bf[0] = [7, 7, 7, 7, 7]
    mant, expo = oracle.quantize(A)
    C, T, _ = oracle.gemm(mant, expo, workloads.fp32_to_bf16_bits(Bf))
    want = np.zeros((M, N))
    want[0] = [2, 4, 6, 8, 10]
    assert np.array_equal(oracle.bf16_to_double(C), want)
    assert np.array_equal(T, np.abs(want))


def test_gemm_identity_and_permutation():
    rng = np.random.default_rng(7)
    K = 64
    A = (rng.standard_normal((48, K)) * np.exp2(rng.integers(-4, 5, size=(48, 1)))).astype(np.float32)
    mant, expo = oracle.quantize(A)
    dec = oracle.decode(mant, expo)
    eye = workloads.fp32_to_bf16_bits(np.eye(K, dtype=np.float32))
    C, _, _ = oracle.gemm(mant, expo, eye)
    assert np.array_equal(oracle.bf16_to_double(C), dec)          # B = I: C = decode(A) exactly
    perm = rng.permutation(K)
    P = np.zeros((K, K), np.float32)
    P[perm, np.arange(K)] = 1.0                                   # column j of C takes column perm[j] of A
    C, _, _ = oracle.gemm(mant, expo, workloads.fp32_to_bf16_bits(P))
    assert np.array_equal(oracle.bf16_to_double(C), dec[:, perm])
    # A = identity (quantises exactly): C = B
    Bb = workloads.fp32_to_bf16_bits(rng.standard_normal((K, 40)).astype(np.float32))
    mi, ei = oracle.quantize(np.eye(K, dtype=np.float32))
    C, _, _ = oracle.gemm(mi, ei, Bb)
    assert np.array_equal(C, Bb)
    # A = row permutation: rows of B permuted
    mi, ei = oracle.quantize(np.eye(K, dtype=np.float32)[perm])
    C, _, _ = oracle.gemm(mi, ei, Bb)
    assert np.array_equal(C, Bb[perm])


def test_gemm_all_ones_counts_k():
    for K in (8, 64, 256):
        mant, expo = oracle.quantize(np.ones((4, K), np.float32))
        C, T, _ = oracle.gemm(mant, expo, workloads.fp32_to_bf16_bits(np.ones((K, 6), np.float32)))
        assert np.all(oracle.bf16_to_double(C) == K) and np.all(T == K)


def test_gemm_small_integers_exact():
    A, Bb = workloads.small_integer_inputs(40, 56, 128, seed=3)
    mant, expo = oracle.quantize(A)
    assert np.array_equal(oracle.decode(mant, expo), A.astype(np.float64))   # lossless for these inputs
    C, _, S, _ = oracle.gemm(mant, expo, Bb, want_sum=True)
    want = A.astype(np.float64) @ workloads.bf16_bits_to_fp32(Bb).astype(np.float64)
    assert np.array_equal(S, want)                                          # integers: exact in any order
    assert np.array_equal(oracle.bf16_to_double(C), oracle.bf16_to_double(oracle.bf16_from_double(want)))


def test_gemm_vs_library_fp64_matmul():
    cfg = workloads.CONFIGS["ragged"]
    A, Bb = workloads.make_inputs(cfg, M=70, N=90, K=264)
    mant, expo = oracle.quantize(A)
    C, T, S, th = oracle.gemm(mant, expo, Bb, want_sum=True)
    assert th >= 1
    dec = oracle.decode(mant, expo)
    Bd = oracle.bf16_to_double(Bb)
    lib = dec @ Bd
    assert np.all(np.abs(S - lib) <= 1e-13 * T + 1e-300)
    assert np.all(np.abs(T - np.abs(dec) @ np.abs(Bd)) <= 1e-13 * T)
    # bf16 result: equal to rounding the library sum except where it sits on a rounding boundary
    same = C == oracle.bf16_from_double(lib)
    assert same.mean() > 0.999
    # selected rows give the same rows
    rows = [69, 0, 13]
    C2, T2, _ = oracle.gemm(mant, expo, Bb, rows=rows)
    assert np.array_equal(C2, C[rows]) and np.array_equal(T2, T[rows])


@pytest.mark.parametrize("tiles", [(32, 64, 64, 64), (64, 64, 64, 64), (8, 32, 16, 48), (16, 128, 24, 32), (1, 7, 8, 5)])
def test_gemm_tiling_invariance(tiles):
    """Walking the ATB nest (C tile -> K-step -> A sub-tile) with one fp64
    accumulator per element visits k in ascending order: bit-identical C for
    every (T_MA, T_MC, T_K, T_N), ragged edges included, and rho*ceil(K/T_K)
    microkernel calls per C tile (Sec. 5)."""
    T_MA, T_MC, T_K, T_N = tiles
    cfg = workloads.CONFIGS["small256"]
    M, N, K = 100, 75, 72
    A, Bb = workloads.make_inputs(cfg, M=M, N=N, K=K)
    mant, expo = oracle.quantize(A)
    C, _, _ = oracle.gemm(mant, expo, Bb)
    Ct, switches = oracle.gemm_tiled(mant, expo, Bb, T_MA, T_MC, T_K, T_N)
    assert np.array_equal(C, Ct)
    n_tiles = -(-M // T_MC) * -(-N // T_N)
    assert switches == n_tiles * (T_MC // T_MA) * -(-K // T_K)


def test_tolerance_formula_value():
    T = np.array([0.0, 128.0])
    assert np.allclose(oracle.tolerance(T), [1e-6, 1.0 + 1e-6], rtol=0, atol=1e-15)
