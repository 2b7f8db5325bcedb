"""Pins for the oracle's bf16 rounding and BFP16 quantise / decode (CPU only).

None of these re-type the oracle's formula: they check it against exact
rational arithmetic, exhaustive enumeration, hand-worked blocks stored as text
and invariants that the definition implies.
"""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------ bf16

def _bf16_value(bits: int) -> Fraction:
    """Exact value of a finite bf16 pattern from the format definition."""
    s = -1 if bits & 0x8000 else 1
    E = (bits >> 7) & 0xFF
    f = bits & 0x7F
    if E == 0:
        return s * Fraction(f, 128) * Fraction(2) ** -126
    return s * (1 + Fraction(f, 128)) * Fraction(2) ** (E - 127)


def _nearest_even_bruteforce(x: Fraction) -> int:
    """Round a rational to bf16 by searching all non-negative finite patterns."""
    ax = abs(x)
    sign = 0x8000 if x < 0 else 0
    best, best_err = None, None
    # patterns are monotone in value: binary search then compare neighbours
    lo, hi = 0, 0x7F7F
    while hi - lo > 1:
        mid = (lo + hi) // 2
        if _bf16_value(mid) <= ax:
            lo = mid
        else:
            hi = mid
    for cand in (lo, hi):
        err = abs(_bf16_value(cand) - ax)
        if best is None or err < best_err or (err == best_err and cand % 2 == 0):
            best, best_err = cand, err
    # overflow threshold: halfway between max finite and 2^128 rounds to inf
    maxf = _bf16_value(0x7F7F)
    if ax >= maxf + (Fraction(2) ** 128 - maxf) / 2:
        best = 0x7F80
    return sign | best


def test_bf16_roundtrip_exhaustive():
    bits = np.arange(0x10000, dtype=np.uint32).astype(np.uint16)
    E = (bits >> 7) & 0xFF
    finite = E != 0xFF
    vals = oracle.bf16_to_double(bits)
    back = oracle.bf16_from_double(vals[finite])
    assert np.array_equal(back, bits[finite])
    # infinities keep their pattern
    assert oracle.bf16_from_double_scalar(float("inf")) == 0x7F80
    assert oracle.bf16_from_double_scalar(float("-inf")) == 0xFF80


def test_bf16_to_double_matches_format_definition():
    rng = np.random.default_rng(1)
    for bits in list(rng.integers(0, 0x7F80, size=300)) + [0, 1, 0x7F, 0x80, 0x7F7F, 0x8001]:
        bits = int(bits)
        assert Fraction(float(oracle.bf16_to_double(np.array([bits], np.uint16))[0])) == _bf16_value(bits)


def test_bf16_midpoints_round_to_even_and_neighbours():
    # every pair of adjacent positive patterns in a spread of binades, incl. subnormals
    starts = [0, 1, 0x7E, 0x7F, 0x80, 0x3F80, 0x3FFF, 0x4000, 0x7F00, 0x7F7E]
    for s in starts:
        for lo in range(s, min(s + 3, 0x7F7F)):
            a, b = _bf16_value(lo), _bf16_value(lo + 1)
            mid = (a + b) / 2
            even = lo if lo % 2 == 0 else lo + 1
            assert oracle.bf16_from_double_scalar(float(mid)) == even          # exact in fp64
            eps = (b - a) / 2 ** 20
            assert oracle.bf16_from_double_scalar(float(mid - eps)) == lo
            assert oracle.bf16_from_double_scalar(float(mid + eps)) == lo + 1
            assert oracle.bf16_from_double_scalar(float(-mid)) == 0x8000 | even


def test_bf16_no_double_rounding():
    # 1 + 2^-8 + 2^-30 lies just above the midpoint of 1 and 1 + 2^-7: must round up.
    # Rounding through fp32 first would land on the midpoint and then go to even (down).
    x = 1.0 + 2.0 ** -8 + 2.0 ** -30
    assert oracle.bf16_from_double_scalar(x) == 0x3F81
    assert oracle.bf16_from_double_scalar(1.0 + 2.0 ** -8) == 0x3F80


def test_bf16_random_vs_bruteforce():
    rng = np.random.default_rng(2)
    xs = np.concatenate([
        rng.standard_normal(300) * np.exp2(rng.integers(-140, 128, size=300)),
        [3.3895e38, 3.4e38, 3.3961775292304601e38, 1e-40, 4.6e-41, 9.2e-41, 2.0 ** -134, 2.0 ** -134 * 1.0001],
    ])
    for x in xs:
        assert oracle.bf16_from_double_scalar(float(x)) == _nearest_even_bruteforce(Fraction(float(x))), x


# ----------------------------------------------------------------- BFP16

def _read_blocks():
    cases, cur = [], {}
    with open(os.path.join(GOLDEN, "bfp16_blocks.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            tag, rest = line.split(None, 1)
            if tag == "x":
                cur = {"x": [eval(tok) for tok in rest.split()]}  # noqa: S307 (our own fixture)
            elif tag == "E":
                cur["E"] = int(rest)
            elif tag == "m":
                cur["m"] = [int(t) for t in rest.split()]
                cases.append(cur)
    return cases


def test_quantize_hand_worked_blocks():
    cases = _read_blocks()
    assert len(cases) >= 6
    for c in cases:
        A = np.array([c["x"]], dtype=np.float32)
        mant, expo = oracle.quantize(A)
        assert int(expo[0, 0]) == c["E"], c
        assert mant[0].tolist() == c["m"], c


def test_quantize_blocks_are_along_k_and_independent():
    rng = np.random.default_rng(3)
    A = rng.standard_normal((5, 32)).astype(np.float32)
    mant, expo = oracle.quantize(A)
    assert mant.shape == (5, 32) and expo.shape == (5, 4)
    # quantising one block alone gives the same bytes: blocks do not interact
    for i in range(5):
        for kb in range(4):
            m1, e1 = oracle.quantize(A[i:i + 1, kb * 8:(kb + 1) * 8])
            assert np.array_equal(m1[0], mant[i, kb * 8:(kb + 1) * 8])
            assert e1[0, 0] == expo[i, kb]


def test_quantize_matches_exact_rational_definition():
    """Brute force: for each block, recompute E and m with Fractions."""
    rng = np.random.default_rng(4)
    A = (rng.standard_normal((16, 64)) * np.exp2(rng.integers(-30, 30, size=(16, 1)))).astype(np.float32)
    A[rng.random(A.shape) < 0.05] *= 256
    A[rng.random(A.shape) < 0.1] = 0
    A[0, :8] = 0
    mant, expo = oracle.quantize(A)
    for i in range(A.shape[0]):
        for kb in range(A.shape[1] // 8):
            xs = [Fraction(float(v)) for v in A[i, kb * 8:(kb + 1) * 8]]
            nz = [abs(v) for v in xs if v != 0]
            if not nz:
                assert expo[i, kb] == 0 and not mant[i, kb * 8:(kb + 1) * 8].any()
                continue
            big = max(nz)
            e = 0
            while Fraction(2) ** (e + 1) <= big:
                e += 1
            while Fraction(2) ** e > big:
                e -= 1
            assert expo[i, kb] == e + 127
            for t, v in enumerate(xs):
                y = v / Fraction(2) ** (e - 6)
                fl = y.numerator // y.denominator
                frac = y - fl
                r = fl + (1 if frac > Fraction(1, 2) or (frac == Fraction(1, 2) and fl % 2 == 1) else 0)
                r = max(-127, min(127, r))
                assert mant[i, kb * 8 + t] == r


def test_quantize_invariants():
    rng = np.random.default_rng(5)
    A = (rng.standard_normal((64, 256)) * np.exp2(rng.integers(-6, 7, size=(64, 1)))).astype(np.float32)
    mant, expo = oracle.quantize(A)
    blk = np.abs(mant.astype(np.int32)).reshape(64, 32, 8).max(axis=2)
    assert blk.min() >= 64 and blk.max() <= 127           # top element normalised into [64, 127]
    dec = oracle.decode(mant, expo)
    # error bound: half a quantum 2^(E-133), one full quantum where the clamp hit
    q = np.exp2(expo.astype(np.float64) - 133.0).repeat(8, axis=1)
    err = np.abs(dec - A.astype(np.float64))
    clamped = np.abs(mant) == 127
    assert np.all(err[~clamped] <= 0.5 * q[~clamped])
    assert np.all(err[clamped] <= 1.0 * q[clamped])
    # idempotent: quantising the decoded values (exact in fp32) reproduces the bytes
    m2, e2 = oracle.quantize(dec.astype(np.float32))
    assert np.array_equal(m2, mant) and np.array_equal(e2, expo)
    # scaling a row by 2^k shifts E by k and leaves the mantissas alone
    for k in (-9, 3, 17):
        m3, e3 = oracle.quantize((A * np.float32(2.0 ** k)).astype(np.float32))
        assert np.array_equal(m3, mant)
        assert np.array_equal(e3.astype(np.int32), expo.astype(np.int32) + k)
    # negation negates the mantissas (symmetric clamp, RNE is symmetric)
    m4, e4 = oracle.quantize(-A)
    assert np.array_equal(m4, -mant) and np.array_equal(e4, expo)


def test_quantize_rejects_bad_input():
    with pytest.raises(ValueError):
        oracle.quantize(np.array([[1, 2, 3, 4, 5, 6, 7, np.inf]], dtype=np.float32))
    with pytest.raises(ValueError):
        oracle.quantize(np.zeros((2, 12), dtype=np.float32))      # K not a multiple of 8


def test_quantize_fp32_subnormal_and_huge():
    tiny = np.float32(2.0 ** -149)
    A = np.array([[tiny, 3 * tiny, 0, 0, 0, 0, 0, 0],
                  [3.0e38, -3.4e38, 1e38, 0, 0, 0, 0, 0]], dtype=np.float32)
    mant, expo = oracle.quantize(A)
    # e = floor(log2(3 * 2^-149)) = -148 -> E clamps to 0 -> m = RNE(x * 2^133): 2^-16 and 3*2^-16 -> 0
    assert expo[0, 0] == 0 and not mant[0].any()
    assert expo[1, 0] == 254                              # 2^127 <= 3.4e38 < 2^128
    dec = oracle.decode(mant, expo)
    assert np.all(np.abs(dec[1, :3] - A[1, :3].astype(np.float64)) <= 2.0 ** (254 - 133))


def test_decode_exhaustive_exact_and_bf16_representable():
    ms = np.arange(-127, 128, dtype=np.int8)
    for E in [0, 1, 6, 7, 8, 100, 127, 133, 200, 254]:
        mant = np.zeros((255, 8), dtype=np.int8)
        mant[:, 3] = ms
        expo = np.full((255, 1), E, dtype=np.uint8)
        dec = oracle.decode(mant, expo)
        for r, m in enumerate(ms):
            assert Fraction(float(dec[r, 3])) == Fraction(int(m)) * Fraction(2) ** (E - 133)
            assert dec[r, 0] == 0.0
        # every decoded value is exactly a bf16 number: the GPU path may decode to bf16 without loss
        bits = oracle.bf16_from_double(dec)
        assert np.array_equal(oracle.bf16_to_double(bits), dec)
