"""Full-size workloads in the launch configuration bench.py times: the whole of C against the oracle
(every element, within the tolerance), every compiled instance against the first bit for bit, plus the
exactness property at full size."""
import time

import numpy as np
import pytest

import oracle
import paper_2511_16041_amd as atb
import workloads
from helpers import bf16_tensor_bits, bits_to_bf16_tensor, unpack_a_bfp

pytestmark = pytest.mark.gpu

# workload -> instances whose whole C is compared with the oracle element by element
CASES = [
    ("square4096", [(256, 256, 64, 256), (128, 256, 64, 256), (64, 256, 64, 256)]),
    ("square8192", [(256, 256, 64, 256), (128, 256, 64, 256), (64, 256, 64, 256), (32, 256, 64, 256), (32, 256, 128, 256)]),
    ("mlp", [(256, 256, 64, 256), (64, 256, 64, 256)]),
    ("ragged", [(256, 256, 64, 256), (64, 256, 64, 256), (32, 64, 64, 64), (32, 256, 128, 256)]),
]
ORACLE_CHUNK = 1024      # rows of C the oracle computes per call (bounds the fp64 temporaries)


def _band_rows(M, rng):
    """Edge rows of the first and last tiles plus one random row out of every 32-row band (the unit a
    wave owns), so that no band of any tile row goes unchecked."""
    edge = [0, 1, 31, 32, 63, 64, 255, 256, M - 257, M - 256, M - 65, M - 33, M - 2, M - 1]
    bands = [min(M - 1, b + int(rng.integers(0, 32))) for b in range(0, M, 32)]
    return np.array(sorted(set([r for r in edge if 0 <= r < M] + bands)), dtype=np.int64)


@pytest.mark.parametrize("name,tile_list", CASES)
def test_full_size_whole_c(name, tile_list):
    """Every element of C, for each listed instance, against the oracle's fp64 result; and every other
    compiled instance bit for bit against the first listed one (all instances add the products of one
    element in the same order, so their roundings agree), which extends the element-wise check to all of them."""
    import torch
    cfg = workloads.CONFIGS[name]
    print(f"full-size {name}: generating", flush=True)
    A, Bb = workloads.make_inputs(cfg)
    M, K = A.shape
    N = Bb.shape[1]
    A_bfp = atb.bfp16_quantize(torch.from_numpy(A).cuda())
    torch.cuda.synchronize()
    lay = atb.bfp16_layout(M, K)
    gm, ge, pad = unpack_a_bfp(A_bfp.cpu().numpy(), M, K, lay)
    print(f"full-size {name}: oracle quantise", flush=True)
    mant, expo = oracle.quantize(A)
    assert np.array_equal(gm, mant) and np.array_equal(ge, expo) and not pad.any()    # quantiser bit-exact at full size
    del A, gm, ge
    B_dev = bits_to_bf16_tensor(Bb, "cuda")
    results = []
    for tiles in tile_list:
        C = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
        g = atb.Gemm(M, N, K, *tiles)
        g.run(A_bfp, B_dev, C)
        torch.cuda.synchronize()
        g.close()
        assert not torch.isnan(C).any().item(), f"{name} {tiles}: unwritten outputs"
        results.append(C)
    first = results[0].view(torch.int16)
    for tiles in atb.instances():
        if tiles in tile_list:
            continue
        C = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
        g = atb.Gemm(M, N, K, *tiles)
        g.run(A_bfp, B_dev, C)
        torch.cuda.synchronize()
        g.close()
        assert torch.equal(C.view(torch.int16), first), f"{name}: instance {tiles} differs from {tile_list[0]}"
        del C
    # bf16 B handed over transposed: same bits as the row-major path, at full size too
    Bt_dev = B_dev.t().contiguous()
    for tiles in tile_list[:2]:
        if tiles[2] != 64:
            continue
        C = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
        g = atb.Gemm(M, N, K, *tiles, b_format="bf16_t")
        g.run(A_bfp, Bt_dev, C)
        torch.cuda.synchronize()
        g.close()
        assert torch.equal(C.view(torch.int16), results[tile_list.index(tiles)].view(torch.int16)), f"{name} {tiles}: transposed-B path differs"
        del C
    del Bt_dev
    t0 = time.perf_counter()
    for r0 in range(0, M, ORACLE_CHUNK):
        r1 = min(M, r0 + ORACLE_CHUNK)
        C_ref, T, _ = oracle.gemm(mant[r0:r1], expo[r0:r1], Bb)
        ref = oracle.bf16_to_double(C_ref)
        tol = oracle.tolerance(T)
        print(f"full-size {name}: oracle rows {r0}..{r1 - 1} after {time.perf_counter() - t0:.1f} s", flush=True)
        for tiles, C in zip(tile_list, results):
            got = oracle.bf16_to_double(bf16_tensor_bits(C[r0:r1]))
            err = np.abs(got - ref)
            assert not (err > tol).any(), f"{name} {tiles} rows {r0}..{r1 - 1}: worst ratio {np.max(err / tol):.3g}"


@pytest.mark.parametrize("name,tiles", [("square4096", (128, 256, 64, 256)), ("square8192", (128, 256, 64, 256)), ("square8192", (256, 256, 64, 256))])
def test_full_size_all_bfp16_sampled_rows(name, tiles):
    """A, B and C stored as BFP16 at full size: sampled rows of the decoded C against the oracle's
    fp64 sums, within the GEMM tolerance plus half a mantissa step of the block."""
    import torch
    cfg = workloads.CONFIGS[name]
    print(f"full-size all-BFP16 {name} {tiles}: generating", flush=True)
    A, Bb = workloads.make_inputs(cfg)
    M, K = A.shape
    N = Bb.shape[1]
    Bt = np.ascontiguousarray(oracle.bf16_to_double(Bb).T.astype(np.float32))
    A_bfp = atb.bfp16_quantize(torch.from_numpy(A).cuda())
    Bt_bfp = atb.bfp16_quantize(torch.from_numpy(Bt).cuda())
    torch.cuda.synchronize()
    mant, expo = oracle.quantize(A)
    bmant, bexpo = oracle.quantize(Bt)
    gm, ge, _ = unpack_a_bfp(Bt_bfp.cpu().numpy(), N, K, atb.bfp16_layout(N, K))
    assert np.array_equal(gm, bmant) and np.array_equal(ge, bexpo)
    del A, Bt, gm, ge
    Bq_bits = np.ascontiguousarray(oracle.bfp16_as_bf16_bits(bmant, bexpo).T)
    rows = _band_rows(M, np.random.default_rng(2))
    print(f"full-size all-BFP16 {name}: oracle gemm on {rows.size} rows", flush=True)
    _, T, S, _ = oracle.gemm(mant, expo, Bq_bits, rows=rows, want_sum=True)
    C = torch.full((atb.bfp16_bytes(M, N),), 0xAB, dtype=torch.uint8, device="cuda")
    g = atb.Gemm(M, N, K, *tiles, b_format="bfp16", c_format="bfp16")
    g.run(A_bfp, Bt_bfp, C)
    torch.cuda.synchronize()
    g.close()
    cm, ce, pad = unpack_a_bfp(C.cpu().numpy(), M, N, atb.bfp16_layout(M, N))
    assert not pad.any()
    val = oracle.decode(cm[rows], ce[rows])
    step = np.repeat(np.ldexp(1.0, ce[rows].astype(np.int64) - 134), 8, axis=1)
    err = np.abs(val - S)
    lim = oracle.tolerance(T) + step
    assert not (err > lim).any(), f"worst ratio {np.max(err / lim):.3g}"


@pytest.mark.parametrize("tiles", [(128, 256, 64, 256), (64, 128, 64, 128)])
def test_b_of_two_gib(tiles):
    """K * N = 2^30: B spans 2^31 bytes, more than a 32-bit signed byte count.  Small-integer inputs make every
    fp32 sum exact, so sampled rows of C must equal the oracle's bit for bit: a B row read from the wrong place,
    or as zero, cannot hide inside a tolerance."""
    import torch
    M, N, K = 300, 32768, 32768
    print(f"B of 2 GiB {tiles}: generating", flush=True)
    rng = np.random.default_rng(21)
    A, _ = workloads.small_integer_inputs(M, 8, K, seed=21)
    lut = workloads.fp32_to_bf16_bits(np.arange(-4, 5, dtype=np.float32))
    # every row of B is different; along N the pattern repeats every 2048 columns (which keeps the generation short)
    Bb = np.tile(lut[rng.integers(0, 9, size=(K, 2048), dtype=np.uint8)], (1, N // 2048))
    mant, expo = oracle.quantize(A)
    rows = np.array([0, 1, 127, 128, 255, 256, 299], dtype=np.int64)
    print(f"B of 2 GiB {tiles}: oracle on {rows.size} rows", flush=True)
    C_ref, _, _ = oracle.gemm(mant, expo, Bb, rows=rows)
    A_bfp = atb.bfp16_quantize(torch.from_numpy(A).cuda())
    B_dev = bits_to_bf16_tensor(Bb, "cuda")
    del Bb
    C = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    g = atb.Gemm(M, N, K, *tiles)
    g.run(A_bfp, B_dev, C)
    torch.cuda.synchronize()
    g.close()
    got = bf16_tensor_bits(C[torch.from_numpy(rows).cuda()])
    assert np.array_equal(got, C_ref)
