// Measurement aid of libatb, not a step of the GEMM: a loop of bf16 MFMAs on register operands with no
// memory traffic at all.  What it sustains is the practical ceiling of the matrix pipes on this chip for
// operands that look like data (the nominal 2.5 PFLOP/s assumes the 2.4 GHz clock, which the chip does not
// hold under full matrix load), so a bench can quote a GEMM against both.  The kernel also reads the two
// wave-visible clocks at its start and end, which tells how fast the shader clock ran under that load.
#include "atb_internal.h"

namespace atb {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kProbeThreads = 512;          // 8 waves, two per SIMD, as the GEMM's large tiles
constexpr int kProbeMfmaPerIter = 32;       // per wave, in units of 32768 flop (one 32 x 32 x 16 MFMA or two 16 x 16 x 32): what one K-step of a 256 x 256 x 64 tile gives a wave

// two bf16 with random sign and mantissa and exponents 2^-7 .. 2 (or the constant 1.0 when `random` is 0)
__device__ __forceinline__ unsigned probe_operand(unsigned &r, int random)
{
    r = r * 1664525u + 1013904223u;
    return random ? ((r & 0x807F807Fu) | 0x3C003C00u | ((r >> 3) & 0x03800380u)) : 0x3F803F80u;
}

// MB = 32: v_mfma_f32_32x32x16_bf16, MB = 16: v_mfma_f32_16x16x32_bf16 (twice as many instructions for the same flop)
template <int MB>
__global__ void __launch_bounds__(kProbeThreads) mfma_probe_kernel(float *sink, unsigned long long *clocks, int iters, int random)
{
    unsigned r = threadIdx.x * 2654435761u + 12345u + blockIdx.x;
    bf16x8 a[4], b[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        union { unsigned u[4]; bf16x8 v; } ua, ub;
#pragma unroll
        for (int e = 0; e < 4; ++e) { ua.u[e] = probe_operand(r, random); ub.u[e] = probe_operand(r, random); }
        a[s] = ua.v;
        b[s] = ub.v;
    }
    constexpr int NACC = (MB == 32) ? 8 : 16, NV = MB * MB / 64, NMFMA = kProbeMfmaPerIter * (32 / MB);
    typedef float accv __attribute__((ext_vector_type(NV)));
    accv acc[NACC];
#pragma unroll
    for (int i = 0; i < NACC; ++i)
#pragma unroll
        for (int v = 0; v < NV; ++v) acc[i][v] = 0.0f;
    const unsigned long long c0 = __builtin_amdgcn_s_memtime(), w0 = __builtin_amdgcn_s_memrealtime();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < NMFMA; ++i) {
            // the operands rotate over four register sets each, so they change from one MFMA to the next
            if constexpr (MB == 32)
                acc[i % NACC] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i % 4], b[(i / 4) % 4], acc[i % NACC], 0, 0, 0);
            else
                acc[i % NACC] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i % 4], b[(i / 4) % 4], acc[i % NACC], 0, 0, 0);
        }
    }
    const unsigned long long c1 = __builtin_amdgcn_s_memtime(), w1 = __builtin_amdgcn_s_memrealtime();
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < NACC; ++i)
#pragma unroll
        for (int q = 0; q < NV; ++q) s += acc[i][q];
    sink[(size_t)blockIdx.x * kProbeThreads + threadIdx.x] = s;
    if (clocks && blockIdx.x == 0 && threadIdx.x == 0) {
        clocks[0] = c1 - c0;      // s_memtime ticks
        clocks[1] = w1 - w0;      // s_memrealtime ticks (constant rate)
    }
}

}  // namespace

hipError_t launch_mfma_probe(float *sink, unsigned long long *clocks, int workgroups, int iters, int random, int mfma_rows, hipStream_t stream)
{
    if (mfma_rows == 32)
        hipLaunchKernelGGL(mfma_probe_kernel<32>, dim3(workgroups), dim3(kProbeThreads), 0, stream, sink, clocks, iters, random);
    else
        hipLaunchKernelGGL(mfma_probe_kernel<16>, dim3(workgroups), dim3(kProbeThreads), 0, stream, sink, clocks, iters, random);
    return hipGetLastError();
}

double mfma_probe_flop(int workgroups, int iters)
{
    return (double)workgroups * (kProbeThreads / 64) * (double)iters * kProbeMfmaPerIter * 32768.0;
}

size_t mfma_probe_sink_bytes(int workgroups) { return (size_t)workgroups * kProbeThreads * sizeof(float); }

}  // namespace atb
