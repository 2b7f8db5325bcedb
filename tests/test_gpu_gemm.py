"""GPU ATB GEMM vs the oracle (runs on an MI355X, through the C ABI).

Acceptance: |C_gpu - C_ref| <= 2^-7 * sum_k |a||b| + 1e-6 for every element;
bit-exact where fp32 accumulation is exact in any order."""
import numpy as np
import pytest

import oracle
import paper_2511_16041_amd as atb
import workloads
from helpers import bf16_tensor_bits, bits_to_bf16_tensor, pack_a_bfp

pytestmark = pytest.mark.gpu

BIG = [(256, 256, 64, 256), (128, 256, 64, 256), (64, 256, 64, 256), (32, 256, 64, 256)]
WIDE_K = [(32, 256, 128, 256)]      # T_K = 128: feasible only with ATB
SMALL = [(64, 64, 64, 64), (32, 64, 64, 64), (64, 64, 128, 128)]
MID = [(128, 128, 64, 256), (64, 128, 64, 256), (128, 128, 64, 128), (64, 128, 64, 128)]
SKINNY = [(32, 64, 256, 64), (32, 32, 256, 64)]      # T_K = 256, a ring of 3 B buffers, helper waves: for problems with one or two rows of C tiles


def _run(mant, expo, Bb, tiles, poison=True):
    import torch
    M, K = mant.shape
    N = Bb.shape[1]
    lay = atb.bfp16_layout(M, K)
    A_dev = torch.from_numpy(pack_a_bfp(mant, expo, lay)).cuda()
    B_dev = bits_to_bf16_tensor(Bb, "cuda")
    C_dev = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda") if poison else None
    g = atb.Gemm(M, N, K, *tiles)
    C_dev = g.run(A_dev, B_dev, C_dev)
    torch.cuda.synchronize()
    g.close()
    return bf16_tensor_bits(C_dev)


def _check(Cg_bits, C_ref, T, what):
    got = oracle.bf16_to_double(Cg_bits)
    assert not np.isnan(got).any(), f"{what}: unwritten or NaN outputs"
    err = np.abs(got - oracle.bf16_to_double(C_ref))
    tol = oracle.tolerance(T)
    bad = err > tol
    assert not bad.any(), f"{what}: {bad.sum()} elements out of tolerance, worst ratio {np.max(err / tol):.3g} at {np.unravel_index(np.argmax(err / tol), err.shape)}"
    return float(np.max(err / tol))


def test_instances_cover_the_tests():
    assert set(BIG + SMALL + MID + WIDE_K + SKINNY) == set(atb.instances())


@pytest.mark.parametrize("tiles", SMALL + SKINNY + MID + BIG + WIDE_K)
def test_small256_config(tiles):
    print(f"gemm small256 tiles={tiles}", flush=True)
    A, Bb = workloads.make_inputs(workloads.CONFIGS["small256"])
    mant, expo = oracle.quantize(A)
    C_ref, T, _ = oracle.gemm(mant, expo, Bb)
    _check(_run(mant, expo, Bb, tiles), C_ref, T, f"small256 {tiles}")


@pytest.mark.parametrize("tiles", SMALL + SKINNY + MID + BIG + WIDE_K)
@pytest.mark.parametrize("shape", [(300, 500, 264), (257, 263, 72), (33, 20, 8), (1, 1, 8), (520, 516, 136), (300, 499, 64), (300, 502, 72), (130, 18, 24)])
def test_ragged_shapes(tiles, shape):
    """Several tiles plus ragged M and N tails, a K tail of 8, N not a multiple of 8, of 4 (rows of B only
    dword-aligned) or of 2 (the element-load variant of the kernel)."""
    M, N, K = shape
    print(f"gemm ragged {shape} tiles={tiles}", flush=True)
    A, Bb = workloads.make_inputs(workloads.CONFIGS["ragged"], M=M, N=N, K=K)
    mant, expo = oracle.quantize(A)
    C_ref, T, _ = oracle.gemm(mant, expo, Bb)
    _check(_run(mant, expo, Bb, tiles), C_ref, T, f"ragged {shape} {tiles}")


@pytest.mark.parametrize("tiles", SMALL + SKINNY + MID + BIG + WIDE_K)
def test_exact_inputs_bitwise(tiles):
    """Small-integer inputs: fp32 accumulation is exact in any order, so every instance
    (every rho) must equal the oracle bit for bit."""
    print(f"gemm exact tiles={tiles}", flush=True)
    A, Bb = workloads.small_integer_inputs(300, 260, 200, seed=5)
    mant, expo = oracle.quantize(A)
    C_ref, _, _ = oracle.gemm(mant, expo, Bb)
    assert np.array_equal(_run(mant, expo, Bb, tiles), C_ref)


@pytest.mark.parametrize("tiles", [(32, 64, 64, 64), (64, 256, 64, 256), (32, 256, 64, 256)])
def test_identity_and_permutation(tiles):
    print(f"gemm identity tiles={tiles}", flush=True)
    rng = np.random.default_rng(11)
    K = 320
    A, _ = workloads.make_inputs(workloads.CONFIGS["mlp"], M=290, N=8, K=K)
    mant, expo = oracle.quantize(A)
    dec = oracle.decode(mant, expo)
    perm = rng.permutation(K)
    P = np.zeros((K, K), np.float32)
    P[perm, np.arange(K)] = 1.0
    got = oracle.bf16_to_double(_run(mant, expo, workloads.fp32_to_bf16_bits(P), tiles))
    assert np.array_equal(got, dec[:, perm])          # decode is exact, products with 1 are exact
    # A = identity: C = B bit for bit
    Bb = workloads.fp32_to_bf16_bits(rng.standard_normal((K, 300)).astype(np.float32))
    mi, ei = oracle.quantize(np.eye(K, dtype=np.float32))
    assert np.array_equal(_run(mi, ei, Bb, tiles), Bb)


def test_deterministic_and_rho_independent():
    """Same kernel twice: bitwise equal.  Different rho at the same C tile and T_K use the same
    per-element accumulation order (k ascending in MFMA slices of 16), so they agree bitwise too."""
    A, Bb = workloads.make_inputs(workloads.CONFIGS["small256"], M=512, N=512, K=512)
    mant, expo = oracle.quantize(A)
    ref = None
    for tiles in BIG:
        c1 = _run(mant, expo, Bb, tiles)
        c2 = _run(mant, expo, Bb, tiles)
        assert np.array_equal(c1, c2)
        if ref is None:
            ref = c1
        assert np.array_equal(ref, c1), tiles


def test_block_exponent_stress():
    """Outliers x2^8 raise the shared exponent (other mantissas underflow), clamped +-127 mantissas,
    zero blocks and large exponent spread inside one row."""
    rng = np.random.default_rng(3)
    M, N, K = 130, 96, 256
    A = rng.standard_normal((M, K)).astype(np.float32)
    A[rng.random((M, K)) < 0.05] *= 256.0
    A[:, 64:72] = 0.0
    A[5] *= np.float32(2.0 ** -20)
    A[6] *= np.float32(2.0 ** 20)
    A[7, ::8] = 3.999
    Bb = workloads.fp32_to_bf16_bits((rng.random((K, N)) * 2 - 1).astype(np.float32))
    mant, expo = oracle.quantize(A)
    assert (np.abs(mant) == 127).any()
    C_ref, T, _ = oracle.gemm(mant, expo, Bb)
    for tiles in [(32, 64, 64, 64), (64, 256, 64, 256)]:
        _check(_run(mant, expo, Bb, tiles), C_ref, T, f"stress {tiles}")


def test_end_to_end_with_gpu_quantizer():
    """fp32 A -> atb_bfp16_quantize -> atb_gemm_run, against oracle quantise + GEMM."""
    import torch
    A, Bb = workloads.make_inputs(workloads.CONFIGS["ragged"], M=300, N=504, K=264)
    mant, expo = oracle.quantize(A)
    C_ref, T, _ = oracle.gemm(mant, expo, Bb)
    A_bfp = atb.bfp16_quantize(torch.from_numpy(A).cuda())
    g = atb.Gemm(300, 504, 264, 64, 256, 64, 256)
    C = g.run(A_bfp, bits_to_bf16_tensor(Bb, "cuda"))
    torch.cuda.synchronize()
    _check(bf16_tensor_bits(C), C_ref, T, "end to end")


def test_run_rejects_bad_arguments():
    import ctypes
    import torch
    g = atb.Gemm(64, 64, 64, 32, 64, 64, 64)
    buf = torch.zeros(4096 * 4, dtype=torch.uint8, device="cuda")
    p = ctypes.c_void_p(buf.data_ptr())
    L = atb.lib()
    assert L.atb_gemm_run(g._h, None, p, p, None) == 1
    assert L.atb_gemm_run(g._h, ctypes.c_void_p(buf.data_ptr() + 2), p, p, None) == 1      # misaligned
    g.close()


@pytest.mark.parametrize("tiles", BIG + WIDE_K)
def test_more_tiles_than_resident_workgroups(tiles):
    """17 x 18 = 306 tiles of 256 x 256 on 256 CUs: the persistent grid gives some workgroups a second
    tile (registers, LDS buffers and in-flight requests of the first must not leak into it), and the
    per-XCD runs of tiles are not a multiple of anything."""
    M, N, K = 4300, 4400, 136
    print(f"gemm persistent {tiles}", flush=True)
    A, Bb = workloads.make_inputs(workloads.CONFIGS["ragged"], M=M, N=N, K=K)
    mant, expo = oracle.quantize(A)
    C_ref, T, _ = oracle.gemm(mant, expo, Bb)
    _check(_run(mant, expo, Bb, tiles), C_ref, T, f"persistent {tiles}")


@pytest.mark.parametrize("tiles", BIG + WIDE_K)
@pytest.mark.parametrize("shape", [(4300, 4400, 8), (4300, 4400, 128), (5900, 5700, 72), (4353, 4609, 200)])
def test_tile_chain_lengths(tiles, shape):
    """A workgroup of the persistent grid runs its tiles as one pipeline: the requests for a tile's first
    operands are issued during the previous tile's last K-steps.  K = 8 and 128 make a tile two K-steps
    long, so the request streams cross a tile boundary inside the prologue and again in every loop body;
    23 x 23 tiles give most workgroups two tiles and some three; the edge tiles are one row or column wide."""
    M, N, K = shape
    print(f"gemm chain {shape} {tiles}", flush=True)
    A, Bb = workloads.make_inputs(workloads.CONFIGS["ragged"], M=M, N=N, K=K)
    mant, expo = oracle.quantize(A)
    C_ref, T, _ = oracle.gemm(mant, expo, Bb)
    _check(_run(mant, expo, Bb, tiles), C_ref, T, f"chain {shape} {tiles}")


@pytest.mark.parametrize("tiles", [(256, 256, 64, 256), (64, 128, 64, 128), (32, 64, 64, 64)])
def test_tile_walk_order_does_not_change_the_result(tiles, monkeypatch):
    """The order in which an XCD's workgroups walk the C tiles (the height of its patch of tiles, which
    the plan reads from ATB_GROUP_M when it is set) decides which tiles share L2, never a value: every
    patch height, also one that does not divide the 17 tile rows, gives the bits of the default."""
    M, N, K = 4300, 4400, 136
    print(f"gemm walk order {tiles}", flush=True)
    A, Bb = workloads.make_inputs(workloads.CONFIGS["ragged"], M=M, N=N, K=K)
    mant, expo = oracle.quantize(A)
    monkeypatch.delenv("ATB_GROUP_M", raising=False)
    base = _run(mant, expo, Bb, tiles)
    C_ref, T, _ = oracle.gemm(mant, expo, Bb)
    _check(base, C_ref, T, f"walk order default {tiles}")
    for rows in ("1", "3", "1000"):
        monkeypatch.setenv("ATB_GROUP_M", rows)
        assert np.array_equal(_run(mant, expo, Bb, tiles), base), f"patch of {rows} tile rows, {tiles}"


def test_graph_capture_and_replay():
    """The run call is a single kernel launch on the caller's stream, so a chain of GEMMs and quantisations can be
    captured into a HIP graph (small problems are launch-bound).  Two layers, y = quantise(x W1) W2, captured once
    and replayed three times with eager work in between; every replay must reproduce the eager result bit for bit."""
    import torch
    M, K, N1, N2 = 200, 264, 256, 136
    A, W1b = workloads.make_inputs(workloads.CONFIGS["small256"], M=M, N=N1, K=K)
    _, W2b = workloads.make_inputs(workloads.CONFIGS["ragged"], M=8, N=N2, K=N1)
    x = atb.bfp16_quantize(torch.from_numpy(A).cuda())
    W1 = bits_to_bf16_tensor(W1b, "cuda")
    W2 = bits_to_bf16_tensor(W2b, "cuda")
    g1 = atb.Gemm(M, N1, K, 32, 64, 64, 64, c_format="bfp16")      # its C is the BFP16 A operand of the second layer
    g2 = atb.Gemm(M, N2, N1, 64, 128, 64, 128)
    h = torch.empty(atb.bfp16_bytes(M, N1), dtype=torch.uint8, device="cuda")
    y = torch.empty((M, N2), dtype=torch.bfloat16, device="cuda")

    def layers():
        g1.run(x, W1, h)
        g2.run(h, W2, y)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        layers()                                # first launches outside the capture (the runtime loads a kernel's code lazily)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    want = bf16_tensor_bits(y)
    print("graph: capturing", flush=True)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        layers()
    for rep in range(3):
        h.fill_(0xAB)
        y.fill_(float("nan"))
        torch.cuda.synchronize()
        print(f"graph: replay {rep}", flush=True)
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(bf16_tensor_bits(y), want), f"replay {rep} differs from the eager result"
    g1.close()
    g2.close()


@pytest.mark.parametrize("tiles", SKINNY + SMALL)
@pytest.mark.parametrize("shape", [(16, 520, 1096), (64, 1030, 2056), (100, 301, 776), (1, 64, 4096)])
def test_skinny_shapes(tiles, shape):
    """Decode-like problems: one or two rows of C tiles, long K (several K-steps of 256 plus a tail of 8)."""
    M, N, K = shape
    print(f"gemm skinny {shape} tiles={tiles}", flush=True)
    A, Bb = workloads.make_inputs(workloads.CONFIGS["mlp"], M=M, N=N, K=K)
    mant, expo = oracle.quantize(A)
    C_ref, T, _ = oracle.gemm(mant, expo, Bb)
    _check(_run(mant, expo, Bb, tiles), C_ref, T, f"skinny {shape} {tiles}")


def test_every_instance_gives_the_same_bits():
    """Tiling changes data movement, not arithmetic: every instance adds the products of an output element in the
    same order (k ascending, 16 per MFMA, one fp32 accumulator), so on any data all instances must agree bit for
    bit -- whatever rho, T_K, wave grid, helper waves or staging variant."""
    shape = (520, 516, 328)
    M, N, K = shape
    print(f"gemm invariance {shape}", flush=True)
    A, Bb = workloads.make_inputs(workloads.CONFIGS["ragged"], M=M, N=N, K=K)
    mant, expo = oracle.quantize(A)
    first = None
    for tiles in atb.instances():
        got = _run(mant, expo, Bb, tiles)
        if first is None:
            first = got
            C_ref, T, _ = oracle.gemm(mant, expo, Bb)
            _check(got, C_ref, T, f"invariance {tiles}")
        else:
            assert np.array_equal(got, first), f"{tiles} differs from {atb.instances()[0]} in {np.count_nonzero(got != first)} elements"


def test_random_shapes_every_instance():
    """Twenty seeded random shapes (M, N <= 700, K <= 1024 in steps of 8, N even and odd) through every instance:
    all instances must agree with each other bit for bit and with the oracle within the tolerance."""
    rng = np.random.default_rng(2024)
    for case in range(20):
        M = int(rng.integers(1, 701))
        N = int(rng.integers(1, 701))
        K = 8 * int(rng.integers(1, 129))
        print(f"gemm random shape {case}: {(M, N, K)}", flush=True)
        A, Bb = workloads.make_inputs(workloads.CONFIGS["ragged"], M=M, N=N, K=K)
        mant, expo = oracle.quantize(A)
        C_ref, T, _ = oracle.gemm(mant, expo, Bb)
        first = None
        for tiles in atb.instances():
            got = _run(mant, expo, Bb, tiles)
            if first is None:
                first = got
                _check(got, C_ref, T, f"random {(M, N, K)} {tiles}")
            else:
                assert np.array_equal(got, first), f"{(M, N, K)}: {tiles} differs from {atb.instances()[0]}"
