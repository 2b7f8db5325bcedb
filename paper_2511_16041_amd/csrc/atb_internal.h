// Internal declarations shared by the translation units of libatb.
// Not part of the public C ABI (see include/atb.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "atb.h"

namespace atb {

// Arguments of one GEMM launch (device pointers are never dereferenced on the host).
struct GemmParams {
    const int8_t *Am;    // mantissa plane  [panels][M][64]
    const uint8_t *Ae;   // exponent plane  [panels][M][8]
    const uint16_t *B;   // bf16 [K][N]                              (B in bf16)
    uint16_t *C;         // bf16 [M][N]                              (C in bf16)
    const int8_t *Bm;    // mantissa plane of B^T  [panels][N][64]   (B in BFP16, blocks along K)
    const uint8_t *Be;   // exponent plane of B^T  [panels][N][8]
    int8_t *Cm;          // mantissa plane of C    [panels of N][M][64]   (C in BFP16, blocks along N)
    uint8_t *Ce;         // exponent plane of C    [panels of N][M][8]
    int M, N, K;
    int k_panels;        // ceil(K / 64): panels of A (and of B^T)
    int n_panels;        // ceil(N / 64): panels of C when it is BFP16
    int tiles_m, tiles_n;   // number of C tiles along M and N
    int group_m;            // tile rows that are walked together (rasterisation)
};

// One compiled kernel instance.
struct Instance {
    int T_MA, T_MC, T_K, T_N;
    int wave_m, wave_n;     // wave grid inside the workgroup
    int threads;            // wave_m * wave_n * 64
    int lds_bytes;          // static LDS of the kernel
    int wg_per_cu;          // workgroups of this instance that share a CU
    int mfma_rows;          // 16: v_mfma_f32_16x16x32_bf16, 32: v_mfma_f32_32x32x16_bf16
    double eff_scale;       // measured full-load throughput of this instance relative to Eq. (12)'s fit; 0: taken from the issue model
    double lone_cap;        // measured largest gain of a workgroup in a sparsely filled round; 0: the default for wg_per_cu
    hipError_t (*launch)(const GemmParams &p, hipStream_t stream);
    bool has_b_transposed;  // launch_fmt also takes b_format = ATB_FMT_BF16_T (with a bf16 C)
    // other storage formats (b_format, c_format as in atb_format); null where the instance has none
    hipError_t (*launch_fmt)(const GemmParams &p, int b_format, int c_format, hipStream_t stream);
};

int instance_count();
const Instance &instance(int i);
// index of the instance with these factors, or -1
int find_instance(int T_MA, int T_MC, int T_K, int T_N);

hipError_t launch_quantize(const float *A, int64_t lda, int8_t *Am, uint8_t *Ae, int64_t M, int64_t K,
                           hipStream_t stream);
hipError_t launch_decode(const int8_t *Am, const uint8_t *Ae, uint16_t *out, int64_t M, int64_t K,
                         hipStream_t stream);
// MFMA-only measurement loop (atb_probe.hip)
hipError_t launch_mfma_probe(float *sink, unsigned long long *clocks, int workgroups, int iters, int random, int mfma_rows, hipStream_t stream);
double mfma_probe_flop(int workgroups, int iters);
size_t mfma_probe_sink_bytes(int workgroups);
constexpr int kPanelK = 64;      // K extent of a panel of the BFP16 layout

static inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

}  // namespace atb
