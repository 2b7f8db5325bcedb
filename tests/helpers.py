"""Test-side helpers: pack oracle BFP16 arrays into the device layout that
include/atb.h documents, and compare a GPU C against the oracle's."""
from __future__ import annotations

import numpy as np


def pack_a_bfp(mant: np.ndarray, expo: np.ndarray, layout) -> np.ndarray:
    """(int8 [M][K], uint8 [M][K/8]) -> uint8 buffer in the planar layout:
    mantissa plane [M][ldm] at 0 (zero padded), exponent plane [M][lde] at exp_off."""
    M, K = mant.shape
    buf = np.zeros(layout.bytes, dtype=np.uint8)
    mp = buf[: M * layout.ldm].reshape(M, layout.ldm)
    mp[:, :K] = mant.view(np.uint8)
    ep = buf[layout.exp_off: layout.exp_off + M * layout.lde].reshape(M, layout.lde)
    ep[:, : K // 8] = expo
    return buf


def unpack_a_bfp(buf: np.ndarray, M: int, K: int, layout):
    mp = buf[: M * layout.ldm].reshape(M, layout.ldm)
    ep = buf[layout.exp_off: layout.exp_off + M * layout.lde].reshape(M, layout.lde)
    return mp[:, :K].view(np.int8).copy(), ep[:, : K // 8].copy(), mp[:, K:].copy()


def bf16_tensor_bits(t) -> np.ndarray:
    """torch bf16 tensor (any device) -> uint16 numpy bit patterns."""
    import torch
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def bits_to_bf16_tensor(bits: np.ndarray, device):
    import torch
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).to(device)
