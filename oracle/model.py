"""Oracle for the analytical model of arXiv 2511.16041 (Secs. 3-5).

TEST INFRASTRUCTURE ONLY: plain Python, written formula by formula from the
paper, used to check the C++ model / tile selector of the GPU library.  It
imports nothing from the product package and the product imports nothing from
here.

Every function names the equation it evaluates.  Byte costs a, b, c are bytes
per element of A, B and C.  Where the paper is inconsistent (it quotes 1.25 B
per BFP16 element in Sec. 3.1 and 9 B per 8 elements in Sec. 2.4) the caller
chooses; tests/test_oracle_model.py shows which value reproduces which column
of Table 2.

What pins what (tests/test_oracle_model.py): Sec. 3 formulas <- Table 2's
columns; Eq. (4) <- the worked example of Sec. 4.1 and brute force over all
issue orders; Eqs. (5), (7), (8), (9) <- a cycle-by-cycle list scheduler (exact
for a single chain, lower bounds otherwise, as the paper states them);
cluster_loads <- the 8 -> 4 example of Sec. 4.2; the chain efficiency of Sec. 5,
Eq. (12) and eff_micro_ilp <- Table 1's Eff_micro column; Eqs. (14), (15) <-
Table 1's trends.  Parity unpinned: Eq. (6) for C > 1 (as printed it falls
below one cycle per VMAC once C > P, the paper prints no value of it, and
Table 1 is met with the one-per-cycle floor binding) and Eq. (10) (checked
only against Eq. (9) algebraically).
"""
from __future__ import annotations

import math
from typing import Sequence, Tuple

# Hardware constants the paper states for the XDNA2 NPU (Secs. 2.4, 3.2, 5).
XDNA2 = {
    "rows": 4,                 # N_aie_row
    "cols": 8,                 # N_aie_col
    "n_core": 32,
    "clock_hz": 1.8e9,
    "mac_per_cycle": 512,      # 8x8x8 BFP16 MAC unit
    "S_L1_bytes": 63 * 1024,
    "bw_offchip": 65e9,
    "delta_cycles": 50.0,
}


def peak_core_flops(mac_per_cycle: float, clock_hz: float) -> float:
    """Sec. 2.4: 512 MAC/cycle * 2 flop * 1.8 GHz = 1.84 TFLOP/s per core."""
    return 2.0 * mac_per_cycle * clock_hz


def ai_rho(T_MC: float, T_N: float, K: float, a: float, b: float, c: float) -> float:
    """Sec. 3.1: AI_rho = 2 / (a/T_N + b/T_MC + c/K)  [op/byte]."""
    return 2.0 / (a / T_N + b / T_MC + c / K)


def ai_rho_from_counts(T_MC, T_K, T_N, K, a, b, c) -> float:
    """Sec. 3.1, first form: operations per output tile / accesses per output
    tile under the output-stationary schedule (N_iterk = K / T_K)."""
    n_iter = K / T_K
    ops = 2.0 * T_MC * T_K * T_N * n_iter
    acc = a * T_MC * T_K * n_iter + b * T_K * T_N * n_iter + c * T_MC * T_N
    return ops / acc


def buffer_bytes(T_MA, T_MC, T_K, T_N, a, b, c) -> float:
    """Eq. (1): (2a/rho) T_MC T_K + 2b T_K T_N + c T_MC T_N, i.e. A and B
    double-buffered, C single-buffered, with rho = T_MC / T_MA."""
    rho = T_MC / T_MA
    return (2.0 * a / rho) * T_MC * T_K + 2.0 * b * T_K * T_N + c * T_MC * T_N


def ai_array(T_MC, T_N, K, a, b, c, rows=4, cols=8) -> float:
    """Eq. (2)-(3): the L2 tile is rows*T_MC x cols*T_N, so
    AI_array = 2 / (a/(cols T_N) + b/(rows T_MC) + c/K)."""
    return 2.0 / (a / (cols * T_N) + b / (rows * T_MC) + c / K)


def t_load(latencies: Sequence[float], counts: Sequence[int], U_LD: int) -> int:
    """Eq. (4): prolog bound.  Sort instruction types by descending latency,
    S_(i) = cumulative count, T_load = max_i (l_(i) + ceil(S_(i)/U_LD) - 1)."""
    order = sorted(range(len(latencies)), key=lambda i: -latencies[i])
    best, S = 0, 0
    for i in order:
        S += counts[i]
        best = max(best, latencies[i] + math.ceil(S / U_LD) - 1)
    return best


def ii_single(P: int, R_load: int, U_LD: int) -> int:
    """Eq. (5): II_single = max(P, ceil(R_load / U_LD))."""
    return max(P, math.ceil(R_load / U_LD))


def ii_parallel(P: int, R_load: int, U_LD: int, C: int) -> float:
    """Eq. (6): II_parallel = max(P + 1 - C, ceil(R_load / U_LD)) / C."""
    return max(P + 1 - C, math.ceil(R_load / U_LD)) / C


def t_steady(II: float, N_accum: int, C: int) -> float:
    """Eq. (7): T_steady >= II_parallel * (N_accum - C)."""
    return II * (N_accum - C)


def t_epilog(l_vmac_vst: int, l_store: int, n_store: int, C: int) -> int:
    """Eq. (8): (l_vmac->vst + l_store + n_store - 1) + (C - 1)."""
    return (l_vmac_vst + l_store + n_store - 1) + (C - 1)


def latency_sequential(T_prolog, T_steady, T_epilog, N_clusters) -> float:
    """Eq. (9): clusters run one after another."""
    return (T_prolog + T_steady + T_epilog) * N_clusters


def latency_overlapped(T_prolog, T_steady, T_epilog, II, C, N_clusters) -> float:
    """Eq. (10): prolog of a cluster hidden under the epilog of the previous."""
    return T_prolog + (T_steady + II * C) * N_clusters + T_epilog


def eff_micro_chain(N_accum, C, T_prolog, II, T_epilog) -> float:
    """Sec. 5, un-numbered: N_accum / (T_prolog + II (N_accum - C) + T_epilog)
    (the N_clusters factor cancels)."""
    return N_accum / (T_prolog + II * (N_accum - C) + T_epilog)


def cluster_loads(rows: int, cols: int, shared: bool) -> int:
    """Sec. 4.2, "Sharing Input Across Chain Cluster": operand loads per
    k-slice of a rows x cols cluster of accumulation chains.  Unshared, each
    of the rows*cols VMACs loads its own A and its own B operand; shared, one
    A operand per cluster row and one B operand per cluster column feed all
    of them."""
    return rows + cols if shared else 2 * rows * cols


# Microbenchmarked parameters of the bfp16ebs8 VMAC that Sec. 4.3 states.
XDNA2_VMAC = {
    "k_per_vmac": 8,       # 8x8x8 MAC unit (Sec. 2.4)
    "n_acc_regs": 5,       # accumulator registers of 8x8 fp32
    "P": 3,                # VMAC pipeline distance
    "l_load": 8,           # operand load latency
    "U_LD": 2,             # vector load units (Sec. 4)
    "l_vmac_vst": 6,
    "l_store": 2,
    "n_store": 2,          # store instructions per accumulator register
}


def eff_micro_ilp(T_K: int, rows: int = 2, cols: int = 2, hw=None) -> float:
    """Microkernel efficiency from the instruction-level model, composed in
    the paper's order: prolog = Eq. (4) over the cluster's operand loads,
    II = Eq. (6), steady state = Eq. (7), epilog = Eq. (8), one cluster after
    another = Eq. (9), efficiency = VMACs issued / cycles (Sec. 4, Sec. 5).

    Readings (the paper leaves them open): the cluster is rows x cols chains
    with shared inputs (Sec. 4.2; 2 x 2 is the example it draws, and the
    largest square cluster that five accumulator registers hold); N_accum
    counts the VMACs of the whole cluster, C * T_K / 8; R_load is the
    cluster's loads per k-slice; and II is floored at one cycle per VMAC,
    because Sec. 4.1 gives every instruction a throughput of one per cycle and
    there is one vector arithmetic unit (Eq. (6) as printed falls below one
    for C > P)."""
    hw = XDNA2_VMAC if hw is None else hw
    C = rows * cols
    loads = cluster_loads(rows, cols, shared=True)
    N_accum = C * (T_K // hw["k_per_vmac"])
    T_prolog = t_load([hw["l_load"]], [loads], hw["U_LD"])
    II = max(1.0, ii_parallel(hw["P"], loads, hw["U_LD"], C))
    T_epi = t_epilog(hw["l_vmac_vst"], hw["l_store"], hw["n_store"], C)
    return eff_micro_chain(N_accum, C, T_prolog, II, T_epi)


def eff_micro(T_K: float, eta: float, eps: float, II: float) -> float:
    """Eq. (12): Eff_micro(T_K) = eta T_K / (eps + eta II T_K)."""
    return eta * T_K / (eps + eta * II * T_K)


def t_asym(T_MC, T_K, T_N, K, rho, peak_core, eff_mic, delta_seconds) -> float:
    """Eq. (14): time for one core to finish one output tile,
    2 T_MC K T_N / (Peak_core Eff_micro) + delta * rho * K / T_K."""
    return 2.0 * T_MC * K * T_N / (peak_core * eff_mic) + delta_seconds * rho * K / T_K


def eff_core(T_MC, T_K, T_N, rho, peak_core, eff_mic, delta_seconds) -> float:
    """Eq. (15): 1 / (1/Eff_micro + delta rho Peak_core / (2 T_MC T_N T_K))."""
    return 1.0 / (1.0 / eff_mic + delta_seconds * rho * peak_core / (2.0 * T_MC * T_N * T_K))


def perf_array(ai: float, bw: float, eff: float, peak_core: float, n_core: int) -> Tuple[float, float, float]:
    """Eq. (11): min(AI * BW_offchip, Eff_core * Peak_core * N_core).
    Returns (perf, memory_bound, compute_bound)."""
    mem = ai * bw
    comp = eff * peak_core * n_core
    return min(mem, comp), mem, comp
