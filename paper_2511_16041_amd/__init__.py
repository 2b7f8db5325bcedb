"""Thin Python binding of libatb (BFP16 x BF16 GEMM with asymmetric tile
buffering for MI355X).  Argument marshalling only: every step of the path runs
in the HIP kernels behind the C ABI declared in include/atb.h.  PyTorch is used
for device memory and streams, nothing else.  There is no CPU fallback: if the
shared library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import List, Optional, Tuple

from . import build as _build

_HERE = os.path.dirname(os.path.abspath(__file__))
_lib = None


class AtbError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().atb_status_string(status).decode()
        extra = f" (hipError {lib().atb_last_hip_error()})" if status == 5 else ""
        super().__init__(f"{where}: {msg}{extra}")


class HwParams(ctypes.Structure):
    _fields_ = [("peak_core_flops", ctypes.c_double), ("n_core", ctypes.c_int),
                ("array_rows", ctypes.c_int), ("array_cols", ctypes.c_int),
                ("bw_offchip", ctypes.c_double), ("buffer_bytes", ctypes.c_double),
                ("acc_bytes", ctypes.c_double), ("clock_hz", ctypes.c_double),
                ("delta_cycles", ctypes.c_double), ("fill_cycles", ctypes.c_double), ("eta", ctypes.c_double),
                ("eps", ctypes.c_double), ("II", ctypes.c_double),
                ("a_bytes", ctypes.c_double), ("b_bytes", ctypes.c_double), ("c_bytes", ctypes.c_double),
                ("a_buf_bytes", ctypes.c_double), ("b_buf_bytes", ctypes.c_double),
                ("n_b_buffers", ctypes.c_int)]


class Choice(ctypes.Structure):
    _fields_ = [("T_MA", ctypes.c_int), ("T_MC", ctypes.c_int), ("T_K", ctypes.c_int), ("T_N", ctypes.c_int),
                ("rho", ctypes.c_int), ("feasible", ctypes.c_int),
                ("ai", ctypes.c_double), ("ai_core", ctypes.c_double),
                ("buffer_bytes", ctypes.c_double), ("acc_bytes", ctypes.c_double),
                ("eff_micro", ctypes.c_double), ("eff_core", ctypes.c_double),
                ("mem_bound", ctypes.c_double), ("compute_bound", ctypes.c_double),
                ("pred_flops", ctypes.c_double)]

    def tiles(self) -> Tuple[int, int, int, int]:
        return (self.T_MA, self.T_MC, self.T_K, self.T_N)


class MicroModel(ctypes.Structure):
    _fields_ = [(n, ctypes.c_double) for n in ("n_mfma", "mfma_cycles", "valu_cycles", "lds_cycles", "vmem_cycles",
                                               "steady_cycles", "switch_cycles", "kstep_cycles", "mfma_util",
                                               "clock_hz", "pred_flops")]


class Bfp16Layout(ctypes.Structure):
    _fields_ = [("panel_k", ctypes.c_int64), ("panels", ctypes.c_int64), ("man_stride", ctypes.c_int64),
                ("exp_stride", ctypes.c_int64), ("exp_off", ctypes.c_int64), ("bytes", ctypes.c_int64)]


# every symbol include/atb.h declares
EXPORTS = [
    "atb_status_string", "atb_last_hip_error", "atb_gemm_create", "atb_gemm_create_fmt", "atb_gemm_run", "atb_gemm_destroy",
    "atb_gemm_launch_info", "atb_instance_count", "atb_instance_get", "atb_bfp16_layout", "atb_bfp16_bytes",
    "atb_bfp16_quantize", "atb_bfp16_decode", "atb_hw_params_xdna2", "atb_hw_params_mi355x",
    "atb_model_eval", "atb_select_tiles", "atb_model_microkernel", "atb_instance_geometry", "atb_mfma_probe",
]


def lib() -> ctypes.CDLL:
    """Load libatb.so (building it if nothing is built); raises if that fails."""
    global _lib
    if _lib is not None:
        return _lib
    path = _build.ensure_built()
    L = ctypes.CDLL(path)
    i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
    pi = ctypes.POINTER(ctypes.c_int)
    L.atb_status_string.restype = ctypes.c_char_p
    L.atb_status_string.argtypes = [ci]
    L.atb_last_hip_error.restype = ci
    L.atb_gemm_create.restype = ci
    L.atb_gemm_create.argtypes = [ctypes.POINTER(vp), i64, i64, i64, ci, ci, ci, ci]
    L.atb_gemm_create_fmt.restype = ci
    L.atb_gemm_create_fmt.argtypes = [ctypes.POINTER(vp), i64, i64, i64, ci, ci, ci, ci, ci, ci]
    L.atb_gemm_run.restype = ci
    L.atb_gemm_run.argtypes = [vp, vp, vp, vp, vp]
    L.atb_gemm_destroy.restype = None
    L.atb_gemm_destroy.argtypes = [vp]
    L.atb_gemm_launch_info.restype = ci
    L.atb_gemm_launch_info.argtypes = [vp, ctypes.POINTER(i64), pi, pi]
    L.atb_instance_count.restype = ci
    L.atb_instance_get.restype = ci
    L.atb_instance_get.argtypes = [ci, pi, pi, pi, pi]
    L.atb_bfp16_layout.restype = ci
    L.atb_bfp16_layout.argtypes = [i64, i64, ctypes.POINTER(Bfp16Layout)]
    L.atb_bfp16_bytes.restype = ctypes.c_size_t
    L.atb_bfp16_bytes.argtypes = [i64, i64]
    L.atb_bfp16_quantize.restype = ci
    L.atb_bfp16_quantize.argtypes = [vp, i64, vp, i64, i64, vp]
    L.atb_bfp16_decode.restype = ci
    L.atb_bfp16_decode.argtypes = [vp, vp, i64, i64, vp]
    L.atb_hw_params_xdna2.restype = None
    L.atb_hw_params_xdna2.argtypes = [ctypes.POINTER(HwParams)]
    L.atb_hw_params_mi355x.restype = None
    L.atb_hw_params_mi355x.argtypes = [ctypes.POINTER(HwParams)]
    L.atb_model_eval.restype = ci
    L.atb_model_eval.argtypes = [i64, i64, i64, ci, ci, ci, ci, ctypes.POINTER(HwParams), ctypes.POINTER(Choice)]
    L.atb_select_tiles.restype = ci
    L.atb_select_tiles.argtypes = [i64, i64, i64, ctypes.POINTER(HwParams), ctypes.POINTER(Choice), ci, pi]
    L.atb_model_microkernel.restype = ci
    L.atb_model_microkernel.argtypes = [ci, ci, ci, ci, ci, ci, ci, ci, ctypes.POINTER(MicroModel)]
    L.atb_instance_geometry.restype = ci
    L.atb_instance_geometry.argtypes = [ci, pi, pi, pi, pi]
    L.atb_mfma_probe.restype = ci
    L.atb_mfma_probe.argtypes = [vp, vp, ci, ci, ci, ci, vp, ctypes.POINTER(ctypes.c_double)]
    _lib = L
    return L


def _check(status: int, where: str) -> None:
    if status != 0:
        raise AtbError(status, where)


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


# ------------------------------------------------------------------ host-only calls

def instances() -> List[Tuple[int, int, int, int]]:
    L = lib()
    out = []
    for i in range(L.atb_instance_count()):
        a, b, c, d = ctypes.c_int(), ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
        _check(L.atb_instance_get(i, a, b, c, d), "atb_instance_get")
        out.append((a.value, b.value, c.value, d.value))
    return out


def bfp16_layout(M: int, K: int) -> Bfp16Layout:
    lay = Bfp16Layout()
    _check(lib().atb_bfp16_layout(M, K, ctypes.byref(lay)), "atb_bfp16_layout")
    return lay


def bfp16_bytes(M: int, K: int) -> int:
    return int(lib().atb_bfp16_bytes(M, K))


def bfp16_pack_host(mant, expo):
    """Host-side layout marshalling (numpy, no arithmetic): (int8 [M][K], uint8 [M][K/8]) -> the uint8
    buffer atb_bfp16_layout(M, K) describes (K-panel-major planes, zero padding)."""
    import numpy as np
    M, K = mant.shape
    lay = bfp16_layout(M, K)
    P, pk = int(lay.panels), int(lay.panel_k)
    buf = np.zeros(lay.bytes, dtype=np.uint8)
    mp = np.zeros((M, P * pk), dtype=np.uint8)
    mp[:, :K] = np.ascontiguousarray(mant).view(np.uint8)
    buf[: P * M * pk] = mp.reshape(M, P, pk).transpose(1, 0, 2).reshape(-1)
    ep = np.zeros((M, P * pk // 8), dtype=np.uint8)
    ep[:, : K // 8] = expo
    buf[lay.exp_off: lay.exp_off + P * M * (pk // 8)] = ep.reshape(M, P, pk // 8).transpose(1, 0, 2).reshape(-1)
    return buf


def bfp16_unpack_host(buf, M: int, K: int):
    """Inverse of bfp16_pack_host: (mant int8 [M][K], expo uint8 [M][K/8], the mantissa bytes of the
    last panel's tail [M][64 * panels - K], which the layout requires to be zero)."""
    import numpy as np
    lay = bfp16_layout(M, K)
    P, pk = int(lay.panels), int(lay.panel_k)
    mp = np.asarray(buf[: P * M * pk]).reshape(P, M, pk).transpose(1, 0, 2).reshape(M, P * pk)
    ep = np.asarray(buf[lay.exp_off: lay.exp_off + P * M * (pk // 8)]).reshape(P, M, pk // 8).transpose(1, 0, 2).reshape(M, P * pk // 8)
    return mp[:, :K].view(np.int8).copy(), ep[:, : K // 8].copy(), mp[:, K:].copy()


def hw_params(which: str = "mi355x") -> HwParams:
    hw = HwParams()
    {"mi355x": lib().atb_hw_params_mi355x, "xdna2": lib().atb_hw_params_xdna2}[which](ctypes.byref(hw))
    return hw


def model_eval(M: int, N: int, K: int, T_MA: int, T_MC: int, T_K: int, T_N: int,
               hw: Optional[HwParams] = None) -> Choice:
    ch = Choice()
    _check(lib().atb_model_eval(M, N, K, T_MA, T_MC, T_K, T_N,
                                ctypes.byref(hw) if hw is not None else None, ctypes.byref(ch)), "atb_model_eval")
    return ch


def instance_geometry(index: int) -> Tuple[int, int, int, int]:
    """(wave_m, wave_n, workgroups per CU, rows of the MFMA form: 16 or 32) of compiled instance `index`."""
    a, b, c, d = ctypes.c_int(), ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
    _check(lib().atb_instance_geometry(index, a, b, c, d), "atb_instance_geometry")
    return a.value, b.value, c.value, d.value


def model_microkernel(T_MA: int, T_MC: int, T_K: int, T_N: int, wave_m: int, wave_n: int, wg_per_cu: int,
                      mfma_rows: int) -> MicroModel:
    m = MicroModel()
    _check(lib().atb_model_microkernel(T_MA, T_MC, T_K, T_N, wave_m, wave_n, wg_per_cu, mfma_rows, ctypes.byref(m)),
           "atb_model_microkernel")
    return m


def select_tiles(M: int, N: int, K: int, hw: Optional[HwParams] = None) -> List[Choice]:
    L = lib()
    n = L.atb_instance_count()
    arr = (Choice * n)()
    cnt = ctypes.c_int()
    _check(L.atb_select_tiles(M, N, K, ctypes.byref(hw) if hw is not None else None, arr, n, ctypes.byref(cnt)),
           "atb_select_tiles")
    return [arr[i] for i in range(min(n, cnt.value))]


# ------------------------------------------------------------------ device calls

def bfp16_quantize(A_f32, stream=None, out=None):
    """A_f32: CUDA fp32 tensor [M][K] (row stride a multiple of 4) -> uint8 tensor holding the A_bfp buffer
    (`out`, if given: a CUDA uint8 tensor of bfp16_bytes(M, K) elements, else a new one)."""
    import torch
    assert A_f32.is_cuda and A_f32.dtype == torch.float32 and A_f32.dim() == 2 and A_f32.stride(1) == 1
    M, K = A_f32.shape
    nbytes = bfp16_bytes(M, K)
    if nbytes == 0:
        raise AtbError(1, "atb_bfp16_bytes")
    if out is None:
        out = torch.empty(nbytes, dtype=torch.uint8, device=A_f32.device)
    assert out.is_cuda and out.dtype == torch.uint8 and out.is_contiguous() and out.numel() == nbytes
    _check(lib().atb_bfp16_quantize(ctypes.c_void_p(A_f32.data_ptr()), A_f32.stride(0),
                                    ctypes.c_void_p(out.data_ptr()), M, K, _stream_ptr(stream)), "atb_bfp16_quantize")
    return out


def bfp16_decode(A_bfp, M: int, K: int, stream=None):
    import torch
    out = torch.empty((M, K), dtype=torch.bfloat16, device=A_bfp.device)
    _check(lib().atb_bfp16_decode(ctypes.c_void_p(A_bfp.data_ptr()), ctypes.c_void_p(out.data_ptr()), M, K,
                                  _stream_ptr(stream)), "atb_bfp16_decode")
    return out


def mfma_probe(sink, clocks, workgroups: int, iters: int, random_operands: bool = True, stream=None, mfma_rows: int = 16) -> float:
    """Launch the MFMA-only measurement loop (atb_mfma_probe).  sink: CUDA float32 tensor of at least
    workgroups * 512 elements; clocks: CUDA int64 tensor of 2 elements, or None; mfma_rows: 16 (16 x 16 x 32 MFMAs, the
    form of the large GEMM tiles) or 32 (32 x 32 x 16).  Returns the launch's flop."""
    import torch
    assert sink.is_cuda and sink.dtype == torch.float32 and sink.numel() >= workgroups * 512
    assert clocks is None or (clocks.is_cuda and clocks.dtype == torch.int64 and clocks.numel() >= 2)
    flop = ctypes.c_double()
    _check(lib().atb_mfma_probe(ctypes.c_void_p(sink.data_ptr()), ctypes.c_void_p(clocks.data_ptr()) if clocks is not None else None,
                                workgroups, iters, 1 if random_operands else 0, mfma_rows, _stream_ptr(stream), ctypes.byref(flop)),
           "atb_mfma_probe")
    return flop.value


@dataclass
class LaunchInfo:
    workgroups: int
    threads: int
    lds_bytes: int


FORMATS = {"bf16": 0, "bfp16": 1, "bf16_t": 2}      # atb_format


class Gemm:
    """A plan from atb_gemm_create / atb_gemm_create_fmt; run() launches it asynchronously.

    b_format "bfp16": run() takes B^T (N x K) as a BFP16 buffer (bfp16_quantize of the N x K matrix);
    b_format "bf16_t": run() takes B^T as a bf16 tensor of shape (N, K);
    c_format "bfp16": run() returns C as a BFP16 buffer with the layout bfp16_layout(M, N)."""

    def __init__(self, M: int, N: int, K: int, T_MA: int, T_MC: int, T_K: int, T_N: int,
                 b_format: str = "bf16", c_format: str = "bf16"):
        self._h = ctypes.c_void_p()
        self.shape = (M, N, K)
        self.tiles = (T_MA, T_MC, T_K, T_N)
        self.b_format, self.c_format = b_format, c_format
        if b_format == "bf16" and c_format == "bf16":
            _check(lib().atb_gemm_create(ctypes.byref(self._h), M, N, K, T_MA, T_MC, T_K, T_N), "atb_gemm_create")
        else:
            _check(lib().atb_gemm_create_fmt(ctypes.byref(self._h), M, N, K, T_MA, T_MC, T_K, T_N,
                                             FORMATS[b_format], FORMATS[c_format]), "atb_gemm_create_fmt")

    def run(self, A_bfp, B, C=None, stream=None):
        import torch
        M, N, K = self.shape
        assert A_bfp.is_cuda and A_bfp.dtype == torch.uint8 and A_bfp.numel() == bfp16_bytes(M, K)
        if self.b_format == "bf16":
            assert B.is_cuda and B.dtype == torch.bfloat16 and tuple(B.shape) == (K, N) and B.is_contiguous()
        elif self.b_format == "bf16_t":
            assert B.is_cuda and B.dtype == torch.bfloat16 and tuple(B.shape) == (N, K) and B.is_contiguous()
        else:
            assert B.is_cuda and B.dtype == torch.uint8 and B.numel() == bfp16_bytes(N, K)
        if self.c_format == "bf16":
            if C is None:
                C = torch.empty((M, N), dtype=torch.bfloat16, device=A_bfp.device)
            assert C.dtype == torch.bfloat16 and tuple(C.shape) == (M, N) and C.is_contiguous()
        else:
            if C is None:
                C = torch.empty(bfp16_bytes(M, N), dtype=torch.uint8, device=A_bfp.device)
            assert C.dtype == torch.uint8 and C.numel() == bfp16_bytes(M, N)
        _check(lib().atb_gemm_run(self._h, ctypes.c_void_p(A_bfp.data_ptr()), ctypes.c_void_p(B.data_ptr()),
                                  ctypes.c_void_p(C.data_ptr()), _stream_ptr(stream)), "atb_gemm_run")
        return C

    def launch_info(self) -> LaunchInfo:
        wg, th, lds = ctypes.c_int64(), ctypes.c_int(), ctypes.c_int()
        _check(lib().atb_gemm_launch_info(self._h, ctypes.byref(wg), ctypes.byref(th), ctypes.byref(lds)),
               "atb_gemm_launch_info")
        return LaunchInfo(wg.value, th.value, lds.value)

    def close(self):
        if self._h:
            lib().atb_gemm_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
