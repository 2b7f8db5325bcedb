"""Test-side helpers: pack oracle BFP16 arrays into the device layout that
include/atb.h documents, and compare a GPU C against the oracle's."""
from __future__ import annotations

import numpy as np


def pack_a_bfp(mant: np.ndarray, expo: np.ndarray, layout=None) -> np.ndarray:
    """(int8 [M][K], uint8 [M][K/8]) -> uint8 buffer in the device layout of include/atb.h,
    written out here independently of the binding's own packer: mantissa plane [panel][row][64]
    at 0 (zero padded), exponent plane [panel][row][8] at exp_off."""
    import paper_2511_16041_amd as atb
    M, K = mant.shape
    lay = atb.bfp16_layout(M, K)
    assert lay.panel_k == 64 and lay.panels == (K + 63) // 64 and lay.man_stride == M * 64 and lay.exp_stride == M * 8
    buf = np.zeros(lay.bytes, dtype=np.uint8)
    mu = mant.view(np.uint8)
    for p in range(int(lay.panels)):
        k0, k1 = 64 * p, min(64 * p + 64, K)
        blk = np.zeros((M, 64), dtype=np.uint8)
        blk[:, : k1 - k0] = mu[:, k0:k1]
        buf[p * lay.man_stride: (p + 1) * lay.man_stride] = blk.reshape(-1)
        eb = np.zeros((M, 8), dtype=np.uint8)
        eb[:, : (k1 - k0) // 8] = expo[:, k0 // 8: k1 // 8]
        buf[lay.exp_off + p * lay.exp_stride: lay.exp_off + (p + 1) * lay.exp_stride] = eb.reshape(-1)
    return buf


def unpack_a_bfp(buf: np.ndarray, M: int, K: int, layout=None):
    """-> (mant int8 [M][K], expo uint8 [M][K/8], mantissa bytes of the last panel's tail)."""
    import paper_2511_16041_amd as atb
    lay = atb.bfp16_layout(M, K)
    P = int(lay.panels)
    mp = np.empty((M, 64 * P), dtype=np.uint8)
    ep = np.empty((M, 8 * P), dtype=np.uint8)
    for p in range(P):
        mp[:, 64 * p: 64 * p + 64] = buf[p * lay.man_stride: (p + 1) * lay.man_stride].reshape(M, 64)
        ep[:, 8 * p: 8 * p + 8] = buf[lay.exp_off + p * lay.exp_stride: lay.exp_off + (p + 1) * lay.exp_stride].reshape(M, 8)
    return mp[:, :K].view(np.int8).copy(), ep[:, : K // 8].copy(), mp[:, K:].copy()


def bf16_tensor_bits(t) -> np.ndarray:
    """torch bf16 tensor (any device) -> uint16 numpy bit patterns."""
    import torch
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def bits_to_bf16_tensor(bits: np.ndarray, device):
    import torch
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).to(device)
