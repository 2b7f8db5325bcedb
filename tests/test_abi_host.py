"""CPU-only tests of libatb: the library loads, exports every symbol the header
declares, validates arguments without touching a device, lays BFP16 out as
documented, and its model / selector agree with the oracle of the paper's model."""
import ctypes

import numpy as np
import os
import re

import pytest

import paper_2511_16041_amd as atb
from oracle import model as om

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "atb.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(atb_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = atb.lib()
    names = _declared_symbols()
    assert len(names) >= 16
    for n in names:
        assert hasattr(L, n), n
    assert sorted(atb.EXPORTS) == names


def test_status_strings():
    L = atb.lib()
    seen = {L.atb_status_string(i) for i in range(7)}
    assert len(seen) == 7 and all(s for s in seen)
    assert L.atb_status_string(99) is not None


def test_instances_and_create_validation():
    inst = atb.instances()
    assert (256, 256, 64, 256) in inst and (64, 256, 64, 256) in inst and (32, 64, 64, 64) in inst
    for (a, c, k, n) in inst:
        assert c % a == 0 and k % 16 == 0
    L = atb.lib()
    h = ctypes.c_void_p()

    def create(M, N, K, *t):
        return L.atb_gemm_create(ctypes.byref(h), M, N, K, *t)

    assert create(256, 256, 256, 32, 64, 64, 64) == 0 and h.value
    wg, th, lds = ctypes.c_int64(), ctypes.c_int(), ctypes.c_int()
    assert L.atb_gemm_launch_info(h, ctypes.byref(wg), ctypes.byref(th), ctypes.byref(lds)) == 0
    assert wg.value == 16 and th.value in (128, 256, 512) and 0 < lds.value <= 160 * 1024
    L.atb_gemm_destroy(h)
    assert create(0, 256, 256, 32, 64, 64, 64) == 1 and not h.value          # M < 1
    assert create(256, 256, 252, 32, 64, 64, 64) == 1                         # K % 8
    assert create(256, 256, 256, 48, 64, 64, 64) == 2                         # T_MC % T_MA
    assert create(256, 256, 256, 64, 64, 32, 64) == 2                         # not compiled
    assert create(256, 256, 256, 512, 512, 64, 256) == 4                      # C tile > accumulators
    assert create(256, 256, 256, 256, 256, 512, 64) == 3                      # A + B > LDS
    assert create(256, 256, 256, 256, 256, 128, 256) == 3                     # T_K = 128 does not fit symmetric ...
    assert create(256, 256, 256, 32, 256, 128, 256) == 0 and h.value         # ... but fits at rho = 8
    L.atb_gemm_destroy(h)
    assert L.atb_gemm_create(None, 1, 1, 8, 32, 64, 64, 64) == 1
    assert L.atb_gemm_run(None, None, None, None, None) == 1
    L.atb_gemm_destroy(None)                                                  # no-op


def test_bfp16_layout():
    for (M, K) in [(256, 256), (3000, 4104), (1, 8), (7, 24)]:
        lay = atb.bfp16_layout(M, K)
        assert lay.panel_k == 64 and lay.panels == (K + 63) // 64
        assert lay.man_stride == M * 64 and lay.exp_stride == M * 8
        assert lay.exp_off % 256 == 0 and lay.exp_off >= lay.panels * lay.man_stride
        assert lay.bytes % 256 == 0 and lay.bytes >= lay.exp_off + lay.panels * lay.exp_stride
        assert atb.bfp16_bytes(M, K) == lay.bytes
    assert atb.bfp16_bytes(4, 12) == 0 and atb.bfp16_bytes(0, 8) == 0
    # 9 bytes per 8 elements, up to padding
    lay = atb.bfp16_layout(8192, 8192)
    assert lay.bytes == 8192 * 8192 * 9 // 8


def test_model_matches_oracle_in_paper_mode():
    hw = atb.hw_params("xdna2")
    assert hw.n_core == 32 and hw.array_rows == 4 and hw.array_cols == 8
    peak = om.peak_core_flops(512, 1.8e9)
    assert hw.peak_core_flops == pytest.approx(peak)
    cases = [(2048, 2048, 4096, 64, 64, 64, 128), (2048, 2048, 4480, 16, 64, 224, 64),
             (4096, 2048, 4096, 32, 128, 64, 128), (4096, 2048, 4096, 128, 128, 8, 128)]
    for (M, N, K, T_MA, T_MC, T_K, T_N) in cases:
        ch = atb.model_eval(M, N, K, T_MA, T_MC, T_K, T_N, hw)
        a, b, c = hw.a_bytes, hw.b_bytes, hw.c_bytes
        rho = T_MC // T_MA
        assert ch.rho == rho
        assert ch.ai_core == pytest.approx(om.ai_rho(T_MC, T_N, K, a, b, c), rel=1e-12)
        assert ch.ai == pytest.approx(om.ai_array(T_MC, T_N, K, a, b, c, 4, 8), rel=1e-12)
        assert ch.buffer_bytes == pytest.approx(om.buffer_bytes(T_MA, T_MC, T_K, T_N, a, b, c), rel=1e-12)
        em = om.eff_micro(T_K, hw.eta, hw.eps, hw.II)
        assert ch.eff_micro == pytest.approx(em, rel=1e-12)
        ec = om.eff_core(T_MC, T_K, T_N, rho, peak, em, hw.delta_cycles / hw.clock_hz)
        assert ch.eff_core == pytest.approx(ec, rel=1e-12)
        perf, mem, comp = om.perf_array(ch.ai, hw.bw_offchip, ec, peak, 32)
        assert ch.mem_bound == pytest.approx(mem, rel=1e-12)
        assert ch.compute_bound == pytest.approx(comp, rel=1e-12)
        assert ch.pred_flops == pytest.approx(perf, rel=1e-12)
        assert ch.feasible == int(ch.buffer_bytes <= 63 * 1024)
    # Table 2, Config 1, 128x64x128 rho=4: AI_array 410, memory bound 26.6 TFLOP/s
    ch = atb.model_eval(4096, 2048, 4096, 32, 128, 64, 128, hw)
    assert round(ch.ai) == 410 and ch.mem_bound / 1e12 == pytest.approx(26.6, abs=0.1)


def test_model_mi355x_mode_and_selector():
    hw = atb.hw_params("mi355x")
    assert hw.n_core == 256 and hw.buffer_bytes == 160 * 1024 and hw.acc_bytes == 256 * 1024
    assert hw.peak_core_flops * hw.n_core == pytest.approx(2.5e15)
    ch = atb.model_eval(8192, 8192, 8192, 64, 256, 64, 256)          # hw = NULL -> MI355X
    ch2 = atb.model_eval(8192, 8192, 8192, 64, 256, 64, 256, hw)
    assert ch.pred_flops == ch2.pred_flops and ch.feasible == 1
    assert ch.acc_bytes == 4 * 256 * 256
    # C lives in registers: the LDS term has no C share
    ab, bb = hw.a_buf_bytes, hw.b_buf_bytes
    assert ch.buffer_bytes == pytest.approx(2 * ab * 64 * 64 + 2 * bb * 64 * 256)
    # Eq. (15) ordering with the fill term switched off: at fixed C tile and T_K, larger rho lowers
    # the compute bound; the LDS footprint always shrinks with rho
    hw0 = atb.hw_params("mi355x")
    hw0.fill_cycles = 0.0
    prev = None
    for T_MA in (256, 128, 64, 32):
        c = atb.model_eval(8192, 8192, 8192, T_MA, 256, 64, 256, hw0)
        if prev is not None:
            assert c.eff_core < prev.eff_core and c.buffer_bytes < prev.buffer_bytes
        prev = c
    # with the fill term: T = T_mfma / Eff_micro + delta rho + fill / rho per K-step
    for T_MA in (256, 128, 64, 32):
        rho = 256 // T_MA
        c = atb.model_eval(8192, 8192, 8192, T_MA, 256, 64, 256, hw)
        t_mfma = 2.0 * 256 * 256 * 64 / hw.peak_core_flops
        t = t_mfma / c.eff_micro + (hw.delta_cycles * rho + hw.fill_cycles / rho) / hw.clock_hz
        assert c.eff_core == pytest.approx(t_mfma / t, rel=1e-12)
    # ATB makes T_K = 128 legal: 264 KiB of LDS symmetric, 146 KiB at rho = 8
    assert atb.model_eval(8192, 8192, 8192, 256, 256, 128, 256, hw).feasible == 0
    assert atb.model_eval(8192, 8192, 8192, 32, 256, 128, 256, hw).feasible == 1
    ranked = atb.select_tiles(8192, 8192, 8192)
    assert len(ranked) == len(atb.instances())
    assert ranked[0].feasible == 1 and ranked[0].T_MC == 256
    assert all(ranked[i].pred_flops >= ranked[i + 1].pred_flops
               for i in range(len(ranked) - 1) if ranked[i + 1].feasible)
    small = atb.select_tiles(256, 256, 256)
    assert small[0].T_MC <= 64                        # many small tiles beat one big tile on 256 CUs
    assert atb.lib().atb_select_tiles(0, 1, 8, None, None, 0, None) == 1


def test_create_fmt_validation():
    """Plans with B and/or C stored as BFP16: argument checks run on the host."""
    L = atb.lib()
    h = ctypes.c_void_p()

    def create(M, N, K, t, bf, cf):
        return L.atb_gemm_create_fmt(ctypes.byref(h), M, N, K, *t, bf, cf)

    assert create(512, 512, 256, (128, 256, 64, 256), 1, 1) == 0 and h.value
    L.atb_gemm_destroy(h)
    assert create(512, 512, 256, (128, 256, 64, 256), 0, 0) == 0 and h.value      # same as atb_gemm_create
    L.atb_gemm_destroy(h)
    assert create(512, 508, 256, (128, 256, 64, 256), 0, 1) == 1 and not h.value  # C in BFP16: N % 8 != 0
    assert create(512, 508, 256, (128, 256, 64, 256), 1, 0) == 0 and h.value      # B in BFP16 does not constrain N
    L.atb_gemm_destroy(h)
    assert create(512, 512, 256, (128, 256, 64, 256), 3, 0) == 1                  # unknown format
    assert create(512, 512, 256, (128, 256, 64, 256), 0, 2) == 1                  # "transposed" is a format of B only
    assert create(512, 508, 256, (128, 256, 64, 256), 2, 0) == 0 and h.value      # bf16 B handed over transposed
    L.atb_gemm_destroy(h)
    assert create(512, 512, 256, (128, 256, 64, 256), 2, 1) == 1                  # ... needs a bf16 C
    assert create(512, 512, 256, (64, 64, 64, 64), 2, 0) == 2                     # ... and one of the large tiles
    assert create(512, 512, 256, (32, 256, 128, 256), 2, 0) == 2
    assert create(64, 64, 1 << 23, (128, 256, 64, 256), 2, 0) == 1                # 2 T_N K >= 2^31
    assert create(512, 512, 256, (32, 256, 64, 256), 0, 1) == 2                   # instance without format variants
    assert create(512, 512, 256, (32, 256, 128, 256), 1, 1) == 2
    assert create(64, 512, 1024, (32, 64, 256, 64), 1, 0) == 0 and h.value           # the skinny-problem instances carry the variants
    L.atb_gemm_destroy(h)
    assert create(512, 512, 256, (64, 64, 64, 64), 1, 1) == 0 and h.value
    L.atb_gemm_destroy(h)


def test_selector_tracks_problem_size():
    """Few C tiles: smaller tiles fill the chip better (the N = 2048 shapes of the paper's Table 3)."""
    assert atb.select_tiles(8192, 8192, 8192)[0].T_MC == 256
    assert atb.select_tiles(4096, 2048, 4096)[0].T_MC == 128         # 128 x 256 and 128 x 128 tiles measure within 3 % of each other here
    assert atb.select_tiles(1024, 2048, 8192)[0].T_MC == 64
    assert atb.select_tiles(1024, 2048, 4096)[0].T_MC <= 128
    assert atb.select_tiles(1024, 2048, 4096)[0].T_N <= 128
    # a launch never beats its fixed cost, and predictions grow with the problem
    a = atb.select_tiles(256, 256, 256)[0].pred_flops
    b = atb.select_tiles(1024, 1024, 1024)[0].pred_flops
    c = atb.select_tiles(8192, 8192, 8192)[0].pred_flops
    assert a < b < c and a < 2.0 * 256 ** 3 / 6e-6


def test_microkernel_model_against_measurements():
    """The CDNA4 issue model (unit costs measured by csrc/microbench/unit_costs.hip) against the
    measured full-load throughput and MFMA-busy fraction of every compiled instance."""
    import os
    rows = []
    for line in open(os.path.join(os.path.dirname(__file__), "measured", "mi355x_instances.txt")):
        if line.startswith("#") or not line.strip():
            continue
        f = line.split()
        rows.append((tuple(int(x) for x in f[:4]), tuple(int(x) for x in f[4:8]), float(f[8]),
                     None if f[9] == "-" else float(f[9]), f[10]))
    inst = atb.instances()
    assert {r[0] for r in rows} == set(inst)
    for tiles, geom, tflops, busy, flag in rows:
        assert atb.instance_geometry(inst.index(tiles)) == geom
        m = atb.model_microkernel(*tiles, *geom)
        # components as documented in include/atb.h
        assert m.n_mfma == tiles[1] * tiles[3] * tiles[2] / 16384 and m.mfma_cycles == m.n_mfma * 8
        assert m.steady_cycles == pytest.approx(max(m.mfma_cycles, m.valu_cycles, m.lds_cycles, m.vmem_cycles) / 0.85)
        assert m.kstep_cycles == pytest.approx(m.steady_cycles + (tiles[1] // tiles[0]) * m.switch_cycles)
        assert m.mfma_util == pytest.approx(m.mfma_cycles / m.kstep_cycles) and 0 < m.mfma_util < 1
        if flag in ("ok", "loose"):
            assert abs(m.pred_flops / 1e12 / tflops - 1) < (0.15 if flag == "ok" else 0.25), (tiles, m.pred_flops / 1e12, tflops)
            if busy is not None:
                # workgroups that share a CU overlap more than the model's division by waves per SIMD grants them:
                # they run busier and at a lower clock than predicted (the throughput bound above still holds)
                assert abs(m.mfma_util - busy) < (0.10 if geom[2] == 1 else 0.15), (tiles, m.mfma_util, busy)
    # every large tile is limited by the VALU issue port (decode next to MFMAs), the small ones by the LDS
    big = atb.model_microkernel(128, 256, 64, 256, 2, 4, 1, 16)
    assert big.valu_cycles > big.mfma_cycles > big.lds_cycles * 0.9 and big.valu_cycles > big.lds_cycles
    small = atb.model_microkernel(64, 64, 64, 64, 2, 2, 4, 16)
    assert small.lds_cycles > small.valu_cycles > small.mfma_cycles
    L = atb.lib()
    assert L.atb_model_microkernel(128, 256, 64, 256, 2, 4, 1, 16, None) == 1
    mm = atb.MicroModel()
    assert L.atb_model_microkernel(96, 256, 64, 256, 2, 4, 1, 16, ctypes.byref(mm)) == 2      # rho not an integer
    assert L.atb_model_microkernel(128, 256, 64, 256, 3, 4, 1, 16, ctypes.byref(mm)) == 2     # bands do not divide


def test_host_packers_agree():
    """The binding's layout marshalling against the tests' own packer (written from include/atb.h)."""
    from helpers import pack_a_bfp, unpack_a_bfp
    rng = np.random.default_rng(0)
    for (M, K) in [(5, 8), (37, 72), (64, 64), (130, 200)]:
        mant = rng.integers(-127, 128, size=(M, K), dtype=np.int8)
        expo = rng.integers(0, 255, size=(M, K // 8), dtype=np.uint8)
        a, b = pack_a_bfp(mant, expo), atb.bfp16_pack_host(mant, expo)
        assert np.array_equal(a, b)
        for unpack in (unpack_a_bfp, atb.bfp16_unpack_host):
            m2, e2, pad = unpack(a, M, K)
            assert np.array_equal(m2, mant) and np.array_equal(e2, expo) and not pad.any()


def test_create_rejects_sizes_beyond_32_bit_offsets():
    """The documented size limits: every operand below 2^31 elements, a B tile's byte offsets below 2^31."""
    import ctypes
    L = atb.lib()
    h = ctypes.c_void_p()
    def create(M, N, K, tiles=(128, 256, 64, 256)):
        return L.atb_gemm_create(ctypes.byref(h), M, N, K, *tiles)
    assert create(256, 32768, 32768) == 0                    # K * N = 2^30 elements: B is 2 GiB, allowed
    L.atb_gemm_destroy(h)
    assert create(256, 65536, 32768) == 1                    # K * N = 2^31
    assert create(65536, 32768, 64) == 1                     # M * N = 2^31
    assert create(32768, 256, 65536) == 1                    # M * K = 2^31
    assert create(64, (1 << 23) + 256, 64) == 1              # N > 2^23
    assert create(64, 1 << 23, 64, (32, 256, 128, 256)) == 1  # 2 N (T_K + 1) >= 2^31 with T_K = 128
    assert create(64, 1 << 23, 64, (128, 256, 64, 256)) == 0
    L.atb_gemm_destroy(h)


def test_selector_against_measured_sweep():
    """The selector's pick against a measured sweep of every instance over 20 problem shapes (large squares, the
    N = 2048 shapes of the paper's Table 3, skinny problems): within 5 % of the fastest instance on each, and the
    predicted throughput of the pick within 30 % of its measurement (20 % but for M = 16)."""
    import os
    inst = atb.instances()
    rows = [l.split() for l in open(os.path.join(os.path.dirname(__file__), "measured", "mi355x_shape_sweep.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 20
    for f in rows:
        M, N, K = (int(x) for x in f[:3])
        meas = [float(x) for x in f[3:]]
        assert len(meas) == len(inst)
        pick = atb.select_tiles(M, N, K)[0]
        got = meas[inst.index(pick.tiles())]
        assert got >= 0.95 * max(meas), ((M, N, K), pick.tiles(), got, inst[meas.index(max(meas))], max(meas))
        assert abs(pick.pred_flops / 1e12 / got - 1) < (0.30 if M < 32 else 0.20), ((M, N, K), pick.tiles(), pick.pred_flops / 1e12, got)
