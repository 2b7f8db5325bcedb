// Analytical model of arXiv 2511.16041 (Secs. 3 and 5) and the tile-factor
// selector built on it.  Pure host arithmetic.
//
//   AI_rho   = 2 / (a/T_N + b/T_MC + c/K)                                  Sec. 3.1
//   buffer   = (2a/rho) T_MC T_K + n_B b T_K T_N + c T_MC T_N <= S         Eq. (1)
//   AI_array = 2 / (a/(cols T_N) + b/(rows T_MC) + c/K)                    Eq. (2)
//   Eff_micro(T_K) = eta T_K / (eps + eta II T_K)                          Eq. (12)
//   Eff_core = 1 / (1/Eff_micro + delta rho Peak_core / (2 T_MC T_N T_K))  Eq. (15)
//              (MI355X: delta rho + fill/rho in place of delta rho, see atb_hw_params.fill_cycles)
//   Perf     = min(AI_array BW, Eff_core Peak_core N_core)                 Eq. (11)
//
// On MI355X the C tile lives in accumulator registers, so Eq. (1) splits in
// two: the A and B terms are charged to the LDS (with the bytes per element
// they occupy there, bf16 after the in-kernel decode) and the C term to the
// accumulator file (fp32).  "rows x cols" is the patch of C tiles that the
// workgroups resident on one XCD share through its L2, the counterpart of the
// 4 x 8 core array that shares L2 tiles by broadcast in the paper.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <vector>

#include "atb_internal.h"

namespace {

// Share of the chip's full-load throughput that `tiles` equal tiles reach when `slots` of them run at a
// time.  Full rounds count 1 each.  A last round that fills only a fraction f of the slots leaves CUs
// (or places on a CU) idle, and its workgroups run faster than in a full round: the chip is power-limited
// under this kernel and clocks the busy CUs higher, and a workgroup with fewer neighbours on its CU has
// more of the CU's issue slots and LDS to itself.  Measured on MI355X (N = 2048 shapes, every instance):
// the gain per workgroup follows f^-3/4 up to a cap that depends on how many workgroups share a CU at full
// load (lone_speedup below); with four or more workgroups per CU it follows 1/f, i.e. a half-filled round of
// small tiles takes half the time.
double round_efficiency(double tiles, double slots, double cap, double exponent = 0.75)
{
    const double full = std::floor(tiles / slots);
    const double f = (tiles - full * slots) / slots;
    double time = full;
    if (f > 0.0) time += 1.0 / std::min(cap, std::pow(f, -exponent));
    return (tiles / slots) / time;
}

// Largest gain of a workgroup in a sparsely filled round over a full one, by workgroups per CU at full
// load: 1.4 for one per CU (the clock alone: 1.33 - 1.39 measured at f = 1/8 .. 1/2), 2.1 for two
// (128 x 128 x 64 x 128 at f = 1/4), 3.0 for three (64 x 128 x 64 x 128 at f = 1/6), about 2 for four and
// more (64 x 64 tiles: 2.0 - 2.1 at f = 1/2 and at f = 1/3).
double lone_speedup(int wg_per_cu)
{
    return wg_per_cu <= 1 ? 1.4 : wg_per_cu == 2 ? 2.1 : wg_per_cu == 3 ? 3.0 : 2.05;
}

// Fixed cost of one launch (measured: a 256^3 problem takes 8 us whatever the tile).
constexpr double kLaunchSeconds = 6.0e-6;

}  // namespace

extern "C" void atb_hw_params_xdna2(atb_hw_params *hw)
{
    if (!hw) return;
    std::memset(hw, 0, sizeof *hw);
    hw->clock_hz = 1.8e9;
    hw->peak_core_flops = 2.0 * 512.0 * 1.8e9;   // 8x8x8 MAC unit, Sec. 2.4
    hw->n_core = 32;
    hw->array_rows = 4;                          // Sec. 3.2
    hw->array_cols = 8;
    hw->bw_offchip = 65e9;                       // Sec. 5
    hw->buffer_bytes = 63.0 * 1024.0;            // Sec. 3.2
    hw->acc_bytes = 0.0;                         // C is buffered in L1
    hw->delta_cycles = 50.0;                     // Sec. 5
    hw->fill_cycles = 0.0;
    hw->eta = 0.03;                              // fitted to Table 1's Eff_micro column
    hw->eps = 1.0;
    hw->II = 1.2;
    hw->a_bytes = 2.0;                           // precision Config 1: A bf16, B BFP16, C bf16
    hw->b_bytes = 1.25;                          // Sec. 3.1 quotes 1.25 B per BFP16 element
    hw->c_bytes = 2.0;
    hw->a_buf_bytes = 0.0;
    hw->b_buf_bytes = 0.0;
    hw->n_b_buffers = 2;
}

extern "C" void atb_hw_params_mi355x(atb_hw_params *hw)
{
    if (!hw) return;
    std::memset(hw, 0, sizeof *hw);
    hw->clock_hz = 2.4e9;
    hw->peak_core_flops = 2.5e15 / 256.0;        // dense bf16 MFMA peak per CU
    hw->n_core = 256;
    hw->array_rows = 8;                          // C tiles co-resident on one XCD (32 CUs): 8 x 4 patch
    hw->array_cols = 4;
    hw->bw_offchip = 8.0e12;                     // HBM3E
    hw->buffer_bytes = 160.0 * 1024.0;           // LDS per CU
    hw->acc_bytes = 256.0 * 1024.0;              // 4 waves x 256 accumulator VGPRs x 64 lanes x 4 B
    // Least-squares fit to the measured K-step times of the 256x256x64 instances at rho = 1, 2, 4, 8
    // on 8192^3 (in cycles of the nominal 2.4 GHz clock): 3417 + 172 rho + 341 / rho, against 2048
    // cycles of MFMA issue, i.e. Eff_micro(64) = 0.599.  T_K = 128 measured no better than 64, so the
    // fit saturates early (small eps): Eff_micro ~ 1 / II.
    hw->delta_cycles = 172.0;
    hw->fill_cycles = 341.0;
    hw->eta = 1.0;
    hw->eps = 0.4;
    hw->II = 1.6620;
    hw->a_bytes = 1.125;                         // A BFP16: 9 bytes per 8 elements
    hw->b_bytes = 2.0;
    hw->c_bytes = 2.0;
    hw->a_buf_bytes = 2.25;                      // decoded bf16 in LDS, 16 B pad per 128 B row
    hw->b_buf_bytes = 2.0;                       // bf16, rows swizzled instead of padded
    hw->n_b_buffers = 2;
}

extern "C" atb_status atb_model_eval(int64_t M, int64_t N, int64_t K, int T_MA, int T_MC, int T_K, int T_N,
                                     const atb_hw_params *hw_in, atb_choice *out)
{
    if (!out || M < 1 || N < 1 || K < 1 || T_MA < 1 || T_MC < 1 || T_K < 1 || T_N < 1) return ATB_ERR_INVALID_ARG;
    if (T_MC % T_MA != 0) return ATB_ERR_BAD_TILE;
    atb_hw_params hw;
    if (hw_in) hw = *hw_in; else atb_hw_params_mi355x(&hw);
    if (hw.peak_core_flops <= 0 || hw.n_core < 1 || hw.array_rows < 1 || hw.array_cols < 1 || hw.clock_hz <= 0 ||
        hw.eta <= 0 || hw.II <= 0)
        return ATB_ERR_INVALID_ARG;

    const double a = hw.a_bytes, b = hw.b_bytes, c = hw.c_bytes;
    const double ab = hw.a_buf_bytes > 0 ? hw.a_buf_bytes : a;
    const double bb = hw.b_buf_bytes > 0 ? hw.b_buf_bytes : b;
    const int nb = hw.n_b_buffers > 0 ? hw.n_b_buffers : 2;
    const double rho = (double)T_MC / (double)T_MA;

    atb_choice r;
    std::memset(&r, 0, sizeof r);
    r.T_MA = T_MA; r.T_MC = T_MC; r.T_K = T_K; r.T_N = T_N;
    r.rho = T_MC / T_MA;
    r.ai_core = 2.0 / (a / T_N + b / T_MC + c / (double)K);
    r.ai = 2.0 / (a / ((double)hw.array_cols * T_N) + b / ((double)hw.array_rows * T_MC) + c / (double)K);
    const bool c_in_regs = hw.acc_bytes > 0.0;
    r.buffer_bytes = (2.0 * ab / rho) * T_MC * T_K + nb * bb * T_K * T_N + (c_in_regs ? 0.0 : c * T_MC * T_N);
    r.acc_bytes = c_in_regs ? 4.0 * T_MC * T_N : 0.0;
    r.feasible = (r.buffer_bytes <= hw.buffer_bytes) && (!c_in_regs || r.acc_bytes <= hw.acc_bytes);
    r.eff_micro = hw.eta * T_K / (hw.eps + hw.eta * hw.II * T_K);
    const double delta_s = hw.delta_cycles / hw.clock_hz;
    const double fill_s = hw.fill_cycles / hw.clock_hz;
    r.eff_core = 1.0 / (1.0 / r.eff_micro +
                        (delta_s * rho + fill_s / rho) * hw.peak_core_flops / (2.0 * T_MC * (double)T_N * T_K));
    r.mem_bound = r.ai * hw.bw_offchip;
    r.compute_bound = r.eff_core * hw.peak_core_flops * hw.n_core;
    if (c_in_regs) {
        // One workgroup per CU at a time: a partly filled last round of tiles idles CUs, and tiles
        // that hang over the matrix edge compute on padding.
        const double tm = std::ceil((double)M / T_MC), tn = std::ceil((double)N / T_N);
        const double useful = ((double)M * (double)N) / (tm * T_MC * tn * T_N);
        r.compute_bound *= round_efficiency(tm * tn, hw.n_core, lone_speedup(1)) * useful;
    }
    r.pred_flops = std::min(r.mem_bound, r.compute_bound);
    if (c_in_regs) {
        const double flop = 2.0 * (double)M * (double)N * (double)K;
        r.pred_flops = flop / (flop / r.pred_flops + kLaunchSeconds);
    }
    *out = r;
    return ATB_OK;
}

// Full-load throughput of an instance relative to what Eqs. (12) and (15) with the 256 x 256 x 64 family's
// constants predict for its tile factors: the microkernel issue model's throughput over that prediction,
// normalised by the same ratio for the symmetric 256 x 256 x 64 x 256 instance (where the fit was made).
double instance_factor(const atb::Instance &x)
{
    auto ratio = [](int T_MA, int T_MC, int T_K, int T_N, int wm, int wn, int wg, int rows) {
        atb_micro_model mm;
        atb_choice ch;
        // a problem large enough that neither round quantisation nor the launch cost matters
        if (atb_model_microkernel(T_MA, T_MC, T_K, T_N, wm, wn, wg, rows, &mm) != ATB_OK ||
            atb_model_eval((int64_t)1 << 20, (int64_t)1 << 20, (int64_t)1 << 16, T_MA, T_MC, T_K, T_N, nullptr, &ch) != ATB_OK ||
            ch.eff_core <= 0.0)
            return 0.0;
        atb_hw_params hw;
        atb_hw_params_mi355x(&hw);
        return mm.pred_flops / (ch.eff_core * hw.peak_core_flops * hw.n_core);
    };
    const double ref = ratio(256, 256, 64, 256, 2, 4, 1, 16);
    const double own = ratio(x.T_MA, x.T_MC, x.T_K, x.T_N, x.wave_m, x.wave_n, x.wg_per_cu, x.mfma_rows);
    return (ref > 0.0 && own > 0.0) ? own / ref : 1.0;
}

extern "C" atb_status atb_select_tiles(int64_t M, int64_t N, int64_t K, const atb_hw_params *hw,
                                       atb_choice *ranked, int capacity, int *count)
{
    if (M < 1 || N < 1 || K < 1 || capacity < 0 || (capacity > 0 && !ranked)) return ATB_ERR_INVALID_ARG;
    try {
    std::vector<atb_choice> all;
    for (int i = 0; i < atb::instance_count(); ++i) {
        const atb::Instance &x = atb::instance(i);
        atb_choice ch;
        atb_status st = atb_model_eval(M, N, K, x.T_MA, x.T_MC, x.T_K, x.T_N, hw, &ch);
        if (st != ATB_OK) return st;
        // Eq. (12) gives Eff_micro as a function of T_K alone, fitted to the 256 x 256 x 64 family.  How far
        // another instance's microkernel deviates from that fit comes from the issue model of the CU
        // (instance_factor below); the few instances that model does not describe carry a measured ratio
        // instead (the paper, too, takes Eff_micro per microkernel from measurement in its Table 1).
        const double scale = x.eff_scale > 0.0 ? x.eff_scale : instance_factor(x);
        ch.compute_bound *= scale;
        ch.eff_core *= scale;
        // the kernels run whole pairs of K-steps: the tail of the last pair multiplies zeros
        ch.compute_bound *= (double)K / (std::ceil((double)K / (2.0 * x.T_K)) * 2.0 * x.T_K);
        atb_hw_params h;
        if (hw) h = *hw; else atb_hw_params_mi355x(&h);
        if ((x.wg_per_cu > 1 || x.lone_cap > 0.0) && h.acc_bytes > 0.0) {
            // several workgroups share a CU, or the instance has a measured cap of its own: redo the round
            // quantisation that atb_model_eval applied for one workgroup per CU
            const double tiles = std::ceil((double)M / x.T_MC) * std::ceil((double)N / x.T_N);
            const double cap = x.lone_cap > 0.0 ? x.lone_cap : lone_speedup(x.wg_per_cu);
            ch.compute_bound *= round_efficiency(tiles, (double)h.n_core * x.wg_per_cu, cap, x.wg_per_cu >= 4 ? 1.0 : 0.75) / round_efficiency(tiles, h.n_core, lone_speedup(1));
        }
        ch.pred_flops = std::min(ch.mem_bound, ch.compute_bound);
        if (h.acc_bytes > 0.0) {
            const double flop = 2.0 * (double)M * (double)N * (double)K;
            ch.pred_flops = flop / (flop / ch.pred_flops + kLaunchSeconds);
        }
        all.push_back(ch);
    }
    std::stable_sort(all.begin(), all.end(), [](const atb_choice &x, const atb_choice &y) {
        if (x.feasible != y.feasible) return x.feasible > y.feasible;
        return x.pred_flops > y.pred_flops;
    });
    if (count) *count = (int)all.size();
    for (int i = 0; i < capacity && i < (int)all.size(); ++i) ranked[i] = all[i];
    return ATB_OK;
    } catch (...) {
        return ATB_ERR_NOMEM;       // the ranking's scratch vector is the only thing here that can throw
    }
}

extern "C" atb_status atb_model_microkernel(int T_MA, int T_MC, int T_K, int T_N, int wave_m, int wave_n,
                                            int wg_per_cu, int mfma_rows, atb_micro_model *out)
{
    if (!out || T_MA < 1 || T_MC < 1 || T_K < 1 || T_N < 1 || wave_m < 1 || wave_n < 1 || wg_per_cu < 1 ||
        (mfma_rows != 16 && mfma_rows != 32))
        return ATB_ERR_INVALID_ARG;
    if (T_MC % T_MA != 0 || T_K % 16 != 0 || T_MC % (32 * wave_m) != 0 || T_N % (32 * wave_n) != 0) return ATB_ERR_BAD_TILE;
    // unit costs, shader-clock cycles (measured, see the header)
    const double kMfmaPipe = 32.0, kMfmaPort = 17.0, kDecodeValu = 6.5, kAddrValu = 4.0;
    const double kReadB128 = 4.7, kReadTr = 4.6, kWriteBytesPerClk = 76.0, kVmemBytesPerClk = 64.0;
    const double kLdsLatency = 120.0, kBarrier = 150.0, kCoIssue = 0.85;
    const double waves = (double)wave_m * wave_n, ks = T_K / 16.0;
    const double mtw = T_MC / 32.0 / wave_m, ntw = T_N / 32.0 / wave_n, rho = (double)T_MC / T_MA;

    atb_micro_model m;
    std::memset(&m, 0, sizeof m);
    m.n_mfma = (double)T_MC * T_N * T_K / (32.0 * 32.0 * 16.0);
    m.mfma_cycles = m.n_mfma * kMfmaPipe / 4.0;
    const double n_decode = 2.5 * T_MC * T_K / 64.0;            // wave instructions: 5 per 2 mantissas per lane
    const double n_addr = 17.0 * waves;                          // descriptor advance, exponent extraction
    m.valu_cycles = (m.n_mfma * kMfmaPort + n_decode * kDecodeValu + n_addr * kAddrValu) / 4.0;
    const double a_reads = waves * mtw * ks;                     // every wave reads its bands' fragments once
    const double b_reads = waves * ks * ntw * 2.0;               // two transposing reads per B fragment
    m.lds_cycles = a_reads * kReadB128 + b_reads * kReadTr + (2.0 * T_MC * T_K + 2.0 * T_K * T_N) / kWriteBytesPerClk;
    m.vmem_cycles = (1.125 * T_MC * T_K + 2.0 * T_K * T_N) / kVmemBytesPerClk;
    m.steady_cycles = std::max(std::max(m.mfma_cycles, m.valu_cycles), std::max(m.lds_cycles, m.vmem_cycles)) / kCoIssue;
    const double waves_per_simd = waves * wg_per_cu / 4.0;
    m.switch_cycles = (kLdsLatency + waves * ks * kReadB128 + kBarrier) / std::max(1.0, waves_per_simd);
    m.kstep_cycles = m.steady_cycles + rho * m.switch_cycles;
    m.mfma_util = m.mfma_cycles / m.kstep_cycles;
    // the 16 x 16 x 32 form of the MFMA draws less power per flop, which the chip turns into clock
    m.clock_hz = std::min(2.4e9, (mfma_rows == 16 ? 1.45e9 : 1.339e9) * std::pow(m.mfma_util, -0.617));
    m.pred_flops = m.n_mfma * 32768.0 * 256.0 / (m.kstep_cycles / m.clock_hz);
    *out = m;
    return ATB_OK;
}

extern "C" atb_status atb_instance_geometry(int index, int *wave_m, int *wave_n, int *wg_per_cu, int *mfma_rows)
{
    if (index < 0 || index >= atb::instance_count()) return ATB_ERR_INVALID_ARG;
    const atb::Instance &x = atb::instance(index);
    if (wave_m) *wave_m = x.wave_m;
    if (wave_n) *wave_n = x.wave_n;
    if (wg_per_cu) *wg_per_cu = x.wg_per_cu;
    if (mfma_rows) *mfma_rows = x.mfma_rows;
    return ATB_OK;
}
