"""B and/or C stored as BFP16 (the all-BFP16 precision configurations of the paper's
Sec. 6.1, with fp32 accumulation) against the oracle, through the C ABI.

B in BFP16 is handed over as B^T (N x K, blocks along K).  Its values are exact bf16 numbers, so the
reference is the same fp64 GEMM on the decoded B.  C in BFP16 is the quantiser's rule applied to the
accumulators: bit-exact against the oracle where fp32 accumulation is exact (small-integer inputs);
otherwise the decoded C must lie within the GEMM tolerance plus half a mantissa step of its block,
(2^-7 * sum|a||b| + 1e-6) + 2^(E - 134), E being the block's stored exponent."""
import numpy as np
import pytest

import oracle
import paper_2511_16041_amd as atb
import workloads
from helpers import bf16_tensor_bits, bits_to_bf16_tensor, pack_a_bfp, unpack_a_bfp

pytestmark = pytest.mark.gpu

FMT_TILES = [(256, 256, 64, 256), (128, 256, 64, 256), (64, 256, 64, 256),
             (128, 128, 64, 256), (64, 128, 64, 256), (128, 128, 64, 128), (64, 128, 64, 128), (64, 64, 64, 64), (32, 64, 64, 64),
             (64, 64, 128, 128), (32, 64, 256, 64), (32, 32, 256, 64)]
COMBOS = [("bfp16", "bf16"), ("bf16", "bfp16"), ("bfp16", "bfp16")]


def _inputs(M, N, K, seed, exact):
    """A fp32 [M][K], B^T fp32 [N][K] (both get quantised), seeded."""
    if exact:
        A, Bb = workloads.small_integer_inputs(M, N, K, seed=seed)
        Bt = np.ascontiguousarray(oracle.bf16_to_double(Bb).T.astype(np.float32))
    else:
        A, Bb = workloads.make_inputs(workloads.CONFIGS["ragged"], M=M, N=N, K=K)
        Bt = np.ascontiguousarray(oracle.bf16_to_double(Bb).T.astype(np.float32))
    return A, Bt


def _reference(A, Bt):
    """(mant, expo, bmant, bexpo, B bits [K][N] of the BFP16-rounded B, C_ref bits, T, S)."""
    mant, expo = oracle.quantize(A)
    bmant, bexpo = oracle.quantize(Bt)
    Bq_bits = np.ascontiguousarray(oracle.bfp16_as_bf16_bits(bmant, bexpo).T)
    return mant, expo, bmant, bexpo, Bq_bits


def _run(mant, expo, B_arg, M, N, K, tiles, b_format, c_format):
    import torch
    A_dev = torch.from_numpy(pack_a_bfp(mant, expo, atb.bfp16_layout(M, K))).cuda()
    if b_format == "bfp16":
        B_dev = torch.from_numpy(pack_a_bfp(B_arg[0], B_arg[1], atb.bfp16_layout(N, K))).cuda()
    else:
        B_dev = bits_to_bf16_tensor(B_arg, "cuda")
    if c_format == "bfp16":
        C_dev = torch.full((atb.bfp16_bytes(M, N),), 0xAB, dtype=torch.uint8, device="cuda")
    else:
        C_dev = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    g = atb.Gemm(M, N, K, *tiles, b_format=b_format, c_format=c_format)
    out = g.run(A_dev, B_dev, C_dev)
    torch.cuda.synchronize()
    g.close()
    if c_format == "bfp16":
        cm, ce, pad = unpack_a_bfp(out.cpu().numpy(), M, N, atb.bfp16_layout(M, N))
        return cm, ce, pad
    return bf16_tensor_bits(out)


@pytest.mark.parametrize("tiles", FMT_TILES)
@pytest.mark.parametrize("fmt", COMBOS)
def test_exact_inputs_bitwise(tiles, fmt):
    b_format, c_format = fmt
    M, N, K = 300, 264, 200
    print(f"formats exact tiles={tiles} B={b_format} C={c_format}", flush=True)
    A, Bt = _inputs(M, N, K, seed=7, exact=True)
    mant, expo, bmant, bexpo, Bq_bits = _reference(A, Bt)
    C_ref, _, S, _ = oracle.gemm(mant, expo, Bq_bits, want_sum=True)
    B_arg = (bmant, bexpo) if b_format == "bfp16" else Bq_bits
    got = _run(mant, expo, B_arg, M, N, K, tiles, b_format, c_format)
    if c_format == "bfp16":
        cm, ce, pad = got
        rm, re_ = oracle.quantize(S.astype(np.float32))      # S is an exact small integer here
        assert np.array_equal(ce, re_) and np.array_equal(cm, rm)
        assert not pad.any(), "row padding of the C mantissa plane must be written as zero"
    else:
        assert np.array_equal(got, C_ref)


@pytest.mark.parametrize("tiles", FMT_TILES)
@pytest.mark.parametrize("fmt", COMBOS)
@pytest.mark.parametrize("shape", [(520, 512, 136), (257, 264, 72), (33, 24, 8), (700, 1032, 320)])
def test_random_inputs(tiles, fmt, shape):
    b_format, c_format = fmt
    M, N, K = shape
    print(f"formats random {shape} tiles={tiles} B={b_format} C={c_format}", flush=True)
    A, Bt = _inputs(M, N, K, seed=3, exact=False)
    mant, expo, bmant, bexpo, Bq_bits = _reference(A, Bt)
    C_ref, T, S, _ = oracle.gemm(mant, expo, Bq_bits, want_sum=True)
    B_arg = (bmant, bexpo) if b_format == "bfp16" else Bq_bits
    got = _run(mant, expo, B_arg, M, N, K, tiles, b_format, c_format)
    tol = oracle.tolerance(T)
    if c_format == "bfp16":
        cm, ce, pad = got
        val = oracle.decode(cm, ce)
        step = np.repeat(np.ldexp(1.0, ce.astype(np.int64) - 134), 8, axis=1)     # half a mantissa step per block
        err = np.abs(val - S)
        bad = err > tol + step
        assert not bad.any(), f"{bad.sum()} elements out of tolerance, worst {np.max(err / (tol + step)):.3g}"
        # the stored exponent is the block maximum's: the largest mantissa of a non-zero block is at least 64
        # unless the block's maximum sits right below a power of two and rounds up into the clamp
        blockmax = np.abs(cm.astype(np.int32)).reshape(M, N // 8, 8).max(axis=2)
        assert np.all((blockmax >= 64) | (ce == 0) | (blockmax == 0)), "exponent larger than the block needs"
        assert not pad.any()
    else:
        err = np.abs(oracle.bf16_to_double(got) - oracle.bf16_to_double(C_ref))
        assert not np.isnan(err).any()
        assert not (err > tol).any(), f"worst ratio {np.max(err / tol):.3g}"


@pytest.mark.parametrize("tiles", [(128, 256, 64, 256), (128, 128, 64, 128), (32, 64, 64, 64)])
@pytest.mark.parametrize("shape", [(300, 263, 72), (129, 502, 136)])
def test_bfp16_b_with_ragged_n(tiles, shape):
    """B in BFP16 does not constrain N (its blocks run along K)."""
    M, N, K = shape
    print(f"formats ragged-N {shape} tiles={tiles}", flush=True)
    A, Bt = _inputs(M, N, K, seed=5, exact=False)
    mant, expo, bmant, bexpo, Bq_bits = _reference(A, Bt)
    C_ref, T, _ = oracle.gemm(mant, expo, Bq_bits)
    got = _run(mant, expo, (bmant, bexpo), M, N, K, tiles, "bfp16", "bf16")
    err = np.abs(oracle.bf16_to_double(got) - oracle.bf16_to_double(C_ref))
    assert not np.isnan(err).any() and not (err > oracle.tolerance(T)).any()


@pytest.mark.parametrize("tiles", [(32, 64, 256, 64), (32, 32, 256, 64)])
@pytest.mark.parametrize("fmt", COMBOS)
@pytest.mark.parametrize("shape", [(16, 520, 776), (64, 264, 1032), (9, 72, 256)])
def test_skinny_problems_with_bfp16_weights(tiles, fmt, shape):
    """Few rows of activations against a wide weight matrix stored as BFP16 (the paper's Config 1 orientation is this
    problem transposed): the instances built for skinny problems, on tiles that lie mostly beyond M."""
    b_format, c_format = fmt
    M, N, K = shape
    print(f"formats skinny {shape} tiles={tiles} B={b_format} C={c_format}", flush=True)
    A, Bt = _inputs(M, N, K, seed=9, exact=False)
    mant, expo, bmant, bexpo, Bq_bits = _reference(A, Bt)
    C_ref, T, S, _ = oracle.gemm(mant, expo, Bq_bits, want_sum=True)
    B_arg = (bmant, bexpo) if b_format == "bfp16" else Bq_bits
    got = _run(mant, expo, B_arg, M, N, K, tiles, b_format, c_format)
    tol = oracle.tolerance(T)
    if c_format == "bfp16":
        cm, ce, pad = got
        step = np.repeat(np.ldexp(1.0, ce.astype(np.int64) - 134), 8, axis=1)
        err = np.abs(oracle.decode(cm, ce) - S)
        assert not (err > tol + step).any(), f"worst {np.max(err / (tol + step)):.3g}"
        assert not pad.any()
    else:
        err = np.abs(oracle.bf16_to_double(got) - oracle.bf16_to_double(C_ref))
        assert not np.isnan(err).any()
        assert not (err > tol).any(), f"worst ratio {np.max(err / tol):.3g}"


BT_TILES = [(256, 256, 64, 256), (128, 256, 64, 256), (64, 256, 64, 256), (128, 128, 64, 256), (64, 128, 64, 256)]


@pytest.mark.parametrize("tiles", BT_TILES)
@pytest.mark.parametrize("shape", [(300, 500, 264), (257, 263, 72), (33, 20, 8), (1, 1, 8), (520, 516, 136), (130, 18, 24),
                                   (700, 1032, 320), (4300, 4400, 136)])
def test_transposed_bf16_b(tiles, shape):
    """bf16 B handed over as B^T (N x K): the same values reach the same MFMAs in the same order, so the result must
    equal the row-major path's bit for bit, besides meeting the oracle's tolerance.  Shapes with ragged M and N, K tails
    that are not whole K-steps (the tile rows of B^T then run into their neighbours, which meet the zero tail of A), a
    single block of K, and more tiles than resident workgroups."""
    import torch
    M, N, K = shape
    print(f"formats transposed-B {shape} tiles={tiles}", flush=True)
    A, Bb = workloads.make_inputs(workloads.CONFIGS["ragged"], M=M, N=N, K=K)
    mant, expo = oracle.quantize(A)
    C_ref, T, _ = oracle.gemm(mant, expo, Bb)
    A_dev = torch.from_numpy(pack_a_bfp(mant, expo, atb.bfp16_layout(M, K))).cuda()
    B_dev = bits_to_bf16_tensor(Bb, "cuda")
    Bt_dev = B_dev.t().contiguous()
    outs = []
    for fmt, Barg in (("bf16", B_dev), ("bf16_t", Bt_dev)):
        C = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
        g = atb.Gemm(M, N, K, *tiles, b_format=fmt)
        g.run(A_dev, Barg, C)
        torch.cuda.synchronize()
        g.close()
        outs.append(bf16_tensor_bits(C))
    err = np.abs(oracle.bf16_to_double(outs[1]) - oracle.bf16_to_double(C_ref))
    assert not np.isnan(err).any()
    assert not (err > oracle.tolerance(T)).any(), f"worst ratio {np.max(err / oracle.tolerance(T)):.3g}"
    assert np.array_equal(outs[0], outs[1]), "transposed-B result differs from the row-major path"


@pytest.mark.parametrize("tiles", BT_TILES)
def test_transposed_bf16_b_exact(tiles):
    import torch
    M, N, K = 300, 264, 200
    A, Bb = workloads.small_integer_inputs(M, N, K, seed=13)
    mant, expo = oracle.quantize(A)
    C_ref, _, _ = oracle.gemm(mant, expo, Bb)
    A_dev = torch.from_numpy(pack_a_bfp(mant, expo, atb.bfp16_layout(M, K))).cuda()
    Bt_dev = bits_to_bf16_tensor(Bb, "cuda").t().contiguous()
    C = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    g = atb.Gemm(M, N, K, *tiles, b_format="bf16_t")
    g.run(A_dev, Bt_dev, C)
    torch.cuda.synchronize()
    g.close()
    assert np.array_equal(bf16_tensor_bits(C), C_ref)


def test_format_argument_errors():
    # C in BFP16 needs whole blocks along N
    with pytest.raises(atb.AtbError) as e:
        atb.Gemm(256, 260, 64, 128, 256, 64, 256, c_format="bfp16")
    assert e.value.status == 1
    # an instance that has no BFP16 B / C variant
    with pytest.raises(atb.AtbError) as e:
        atb.Gemm(256, 256, 64, 32, 256, 64, 256, c_format="bfp16")
    assert e.value.status == 2


@pytest.mark.parametrize("tiles", [(128, 256, 64, 256), (64, 64, 64, 64)])
def test_bfp16_output_feeds_the_next_gemm(tiles):
    """Two layers: C1 = A x B1 written as BFP16, then C2 = C1 x B2 with C1 taken as it is (its row
    padding included) as the BFP16 operand.  Small-integer inputs make the first stage's sums exact, so the
    oracle's own C1 codes equal the GPU's (asserted); stage 2 then has identical inputs on both sides and must
    meet the GEMM tolerance."""
    import torch
    M, N1, K1, N2 = 300, 264, 200, 136
    print(f"formats chain tiles={tiles}", flush=True)
    A, B1 = workloads.small_integer_inputs(M, N1, K1, seed=11)
    _, B2 = workloads.small_integer_inputs(8, N2, N1, seed=12)             # bf16 bits [N1][N2]
    mant, expo = oracle.quantize(A)
    _, _, S1, _ = oracle.gemm(mant, expo, B1, want_sum=True)
    c1m, c1e = oracle.quantize(S1.astype(np.float32))
    C2_ref, T2, _ = oracle.gemm(c1m, c1e, B2)

    A_dev = torch.from_numpy(pack_a_bfp(mant, expo, atb.bfp16_layout(M, K1))).cuda()
    g1 = atb.Gemm(M, N1, K1, *tiles, c_format="bfp16")
    C1_dev = g1.run(A_dev, bits_to_bf16_tensor(B1, "cuda"), torch.full((atb.bfp16_bytes(M, N1),), 0xAB, dtype=torch.uint8, device="cuda"))
    g2 = atb.Gemm(M, N2, N1, *tiles)
    C2_dev = g2.run(C1_dev, bits_to_bf16_tensor(B2, "cuda"))
    torch.cuda.synchronize()
    g1.close(); g2.close()
    gm, ge, pad = unpack_a_bfp(C1_dev.cpu().numpy(), M, N1, atb.bfp16_layout(M, N1))
    assert np.array_equal(gm, c1m) and np.array_equal(ge, c1e) and not pad.any()
    err = np.abs(oracle.bf16_to_double(bf16_tensor_bits(C2_dev)) - oracle.bf16_to_double(C2_ref))
    assert not np.isnan(err).any() and not (err > oracle.tolerance(T2)).any()


@pytest.mark.parametrize("tiles", [(256, 256, 64, 256), (128, 256, 64, 256), (64, 256, 64, 256)])
@pytest.mark.parametrize("fmt", COMBOS)
@pytest.mark.parametrize("shape", [(4300, 4400, 8), (4600, 4360, 136)])
def test_formats_across_tile_boundaries(tiles, fmt, shape):
    """More 256 x 256 tiles than resident workgroups: the BFP16 B stream (three K-steps ahead) and the
    BFP16 epilogue run across the boundaries between a workgroup's tiles."""
    b_format, c_format = fmt
    M, N, K = shape
    print(f"formats chain {shape} tiles={tiles} B={b_format} C={c_format}", flush=True)
    A, Bt = _inputs(M, N, K, seed=5, exact=False)
    mant, expo, bmant, bexpo, Bq_bits = _reference(A, Bt)
    C_ref, T, S, _ = oracle.gemm(mant, expo, Bq_bits, want_sum=True)
    B_arg = (bmant, bexpo) if b_format == "bfp16" else Bq_bits
    got = _run(mant, expo, B_arg, M, N, K, tiles, b_format, c_format)
    tol = oracle.tolerance(T)
    if c_format == "bfp16":
        cm, ce, pad = got
        step = np.repeat(np.ldexp(1.0, ce.astype(np.int64) - 134), 8, axis=1)
        err = np.abs(oracle.decode(cm, ce) - S)
        assert not (err > tol + step).any(), f"worst {np.max(err / (tol + step)):.3g}"
        assert not pad.any()
    else:
        err = np.abs(oracle.bf16_to_double(got) - oracle.bf16_to_double(C_ref))
        assert not np.isnan(err).any()
        assert not (err > tol).any(), f"worst ratio {np.max(err / tol):.3g}"
