"""GPU BFP16 quantiser / decoder vs the oracle: bit-exact (runs on an MI355X)."""
import numpy as np
import pytest

import oracle
import paper_2511_16041_amd as atb
import workloads
from helpers import bf16_tensor_bits, unpack_a_bfp

pytestmark = pytest.mark.gpu


def _quantize_gpu(A):
    import torch
    At = torch.from_numpy(A).cuda()
    buf = atb.bfp16_quantize(At)
    torch.cuda.synchronize()
    M, K = A.shape
    lay = atb.bfp16_layout(M, K)
    return buf, unpack_a_bfp(buf.cpu().numpy(), M, K, lay)


@pytest.mark.parametrize("name,M,K", [("small256", 256, 256), ("ragged", 300, 264), ("ragged", 37, 4104),
                                      ("mlp", 129, 1024), ("small256", 1, 8), ("ragged", 5, 24)])
def test_quantizer_bit_exact(name, M, K):
    print(f"quantize {name} M={M} K={K}", flush=True)
    A, _ = workloads.make_inputs(workloads.CONFIGS[name], M=M, N=8, K=K)
    mant, expo = oracle.quantize(A)
    _, (gm, ge, pad) = _quantize_gpu(A)
    assert np.array_equal(ge, expo)
    assert np.array_equal(gm, mant)
    assert not pad.any()                       # mantissa padding is zero


def test_quantizer_special_blocks():
    """Zero blocks, ties, saturation to +-127, tiny and huge exponents."""
    rows = [
        [1.0, 0.5, -0.75, 2 ** -7, 1.5 * 2 ** -7, 255 / 128, -1.0, 0.0],
        [1.0, 1.5 / 64, 2.5 / 64, 3.5 / 64, -0.5 / 64, -1.5 / 64, 0.0, 0.0],
        [0.0, -0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0],
        [256.0, 1.0, -1.0, 1.9, 2.0, -3.0, 0.99, 0.0],
        [3.999, -3.999, 2.0, 0.03125, 0.0, 0.0, 0.0, 0.0],
        [3.0e38, -3.4e38, 1e38, 0, 0, 0, 0, 0],
        [1e-30, -3e-31, 2e-32, 0, 0, 0, 0, 1e-35],
        [1.17549435e-38, 1e-38, -1.2e-38, 0, 0, 0, 0, 0],          # around the smallest normal fp32
    ]
    A = np.array(rows, dtype=np.float32)
    A = np.concatenate([A, A[:, ::-1]], axis=1)                    # two blocks per row
    mant, expo = oracle.quantize(A)
    _, (gm, ge, _) = _quantize_gpu(A)
    assert np.array_equal(ge, expo) and np.array_equal(gm, mant)


def test_quantizer_row_pitch():
    import torch
    A, _ = workloads.make_inputs(workloads.CONFIGS["small256"], M=33, N=8, K=72)
    big = torch.zeros((33, 80), dtype=torch.float32, device="cuda")
    big[:, :72] = torch.from_numpy(A).cuda()
    buf = atb.bfp16_quantize(big[:, :72])                          # lda = 80
    torch.cuda.synchronize()
    gm, ge, _ = unpack_a_bfp(buf.cpu().numpy(), 33, 72, atb.bfp16_layout(33, 72))
    mant, expo = oracle.quantize(A)
    assert np.array_equal(ge, expo) and np.array_equal(gm, mant)


def test_decode_exact():
    import torch
    A, _ = workloads.make_inputs(workloads.CONFIGS["ragged"], M=70, N=8, K=264)
    mant, expo = oracle.quantize(A)
    buf, _ = _quantize_gpu(A)
    dec = atb.bfp16_decode(buf, 70, 264)
    torch.cuda.synchronize()
    got = oracle.bf16_to_double(bf16_tensor_bits(dec))
    assert np.array_equal(got, oracle.decode(mant, expo))


def test_quantizer_rejects_bad_arguments():
    import ctypes
    import torch
    L = atb.lib()
    A = torch.zeros((4, 16), dtype=torch.float32, device="cuda")
    out = torch.zeros(atb.bfp16_bytes(4, 16), dtype=torch.uint8, device="cuda")
    p = lambda t: ctypes.c_void_p(t.data_ptr())
    assert L.atb_bfp16_quantize(p(A), 16, p(out), 4, 12, None) == 1      # K % 8
    assert L.atb_bfp16_quantize(p(A), 8, p(out), 4, 16, None) == 1       # lda < K
    assert L.atb_bfp16_quantize(None, 16, p(out), 4, 16, None) == 1
    assert L.atb_bfp16_quantize(ctypes.c_void_p(A.data_ptr() + 4), 16, p(out), 4, 16, None) == 1   # misaligned
