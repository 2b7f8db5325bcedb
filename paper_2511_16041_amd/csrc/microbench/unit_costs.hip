// Unit costs of the gfx950 CU that the CDNA4 microkernel model (atb_model_microkernel) is built
// from: how long an 8-pass MFMA holds the matrix pipe and the SIMD's VALU issue port, what another
// VALU instruction costs next to it, and what the LDS charges for the three access kinds of the
// GEMM kernel.  Developer tool, not part of libatb: build with
//     hipcc --offload-arch=gfx950 -O3 -std=c++17 -Xclang -target-feature -Xclang -packed-fp32-ops -o unit_costs unit_costs.hip
// and run on the GPU; it prints one line per experiment.  Every kernel runs one 512-thread workgroup
// per CU (two waves per SIMD, as the GEMM does), a fixed number of iterations, and touches only its own
// LDS and one output word per thread.  It prints nanoseconds; run it under
//     rocprofv3 --pmc GRBM_GUI_ACTIVE --output-format csv -d <dir> -o p -- ./unit_costs
// as well: GRBM_GUI_ACTIVE / 8 of a dispatch is its length in shader clocks (the clock depends on the
// load, so each experiment has its own), which turns the figures into cycles.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef int intx4 __attribute__((ext_vector_type(4)));
typedef short shortx4 __attribute__((ext_vector_type(4)));

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); exit(1); } } while (0)
#define FENCE() __builtin_amdgcn_sched_barrier(0)

constexpr int kThreads = 512, kBlocks = 256, kLds = 64 * 1024;

__device__ __forceinline__ float byte_to_float(int w, int b) { return (float)(int)(signed char)(w >> (8 * b)); }

// MODE 0: 8 MFMAs per iteration, each followed by PAIRS BFP16 decode pairs (2 cvt, 2 ldexp, 1 pack).
// MODE 1: 8 b128 fragment reads per iteration (lane l: row l % 32 at pitch 144, k half l / 32).
// MODE 2: 8 transposing b64 reads per iteration (the swizzled B-tile pattern of the GEMM).
// MODE 3: 8 b128 writes per iteration (the A staging pattern: 4 lanes per row of pitch 144).
// MODE 4: MODE 0 with pseudo-random bf16 operands (random sign and mantissa, exponents 2^-7 .. 2): the
//         matrix pipes draw more power than on constants, and the chip answers with a lower clock.
template <int MODE, int PAIRS>
__global__ void __launch_bounds__(kThreads) cost_kernel(float *out, int iters, int seed)
{
    __shared__ __attribute__((aligned(16))) char lds[kLds];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    for (int i = t; i < kLds / 4; i += kThreads) reinterpret_cast<int *>(lds)[i] = i * seed;
    __syncthreads();
    bf16x8 a, b;
    for (int e = 0; e < 8; ++e) { a[e] = (__bf16)(float)((t + e) % 3); b[e] = (__bf16)(float)((t + e) % 5); }
    if (MODE == 4) {
        union { unsigned u[4]; bf16x8 v; } ua, ub;
        unsigned r = t * 2654435761u + 12345u;
        for (int e = 0; e < 4; ++e) {
            r = r * 1664525u + 1013904223u; ua.u[e] = (r & 0x807F807Fu) | 0x3C003C00u | ((r >> 3) & 0x03800380u);
            r = r * 1664525u + 1013904223u; ub.u[e] = (r & 0x807F807Fu) | 0x3C003C00u | ((r >> 3) & 0x03800380u);
        }
        a = ua.v; b = ub.v;
    }
    floatx16 acc[8];
    for (int i = 0; i < 8; ++i) for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    int w0 = seed + t, sh = seed & 3;
    unsigned dsum = 0;
    intx4 rsum = {0, 0, 0, 0};
    const char *frag = lds + (wave & 3) * 4608 + (lane & 31) * 144 + (lane >> 5) * 16;           // < 18.5 KiB + 4.7 KiB
    const char *frag_alt = lds + ((wave + 1) & 3) * 4608 + (lane & 31) * 144 + (lane >> 5) * 16;
    const int blk = lane >> 4, j = lane & 15, r = j >> 2;
    const char *tr = lds + 24576 + (8 * (blk >> 1) + r) * 512 + (((4 * (wave & 3) + 2 * (blk & 1) + ((j & 3) >> 1)) ^ (r << 2)) * 16) + (j & 1) * 8;   // 16 rows x 512 B
    char *wr = lds + 36864 + (t >> 2) * 144 + (t & 3) * 32;                                        // 128 rows x 144 B
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (MODE == 0 || MODE == 4) {
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
                FENCE();
#pragma unroll
                for (int v = 0; v < PAIRS; ++v) {
                    const float f0 = ldexpf(byte_to_float(w0, (2 * v) & 3), sh), f1 = ldexpf(byte_to_float(w0, (2 * v + 1) & 3), sh);
                    union { bf16x2 p; unsigned u; } pk;
                    pk.p = bf16x2{(__bf16)f0, (__bf16)f1};
                    dsum ^= pk.u;
                    w0 += 0x01010101;
                }
                FENCE();
            } else if (MODE == 1) {
                rsum += *reinterpret_cast<const intx4 *>(((i >> 2) ? frag_alt : frag) + (i & 3) * 32);
                asm volatile("" ::: "memory");
            } else if (MODE == 2) {
                typedef __attribute__((address_space(3))) shortx4 lds_shortx4;
                const shortx4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_shortx4 *)(tr + (i & 1) * 2048 + ((i >> 1) & 1) * 256));
                rsum.x += v[0]; rsum.y += v[3];
                asm volatile("" ::: "memory");
            } else {
                *reinterpret_cast<intx4 *>(wr + (i & 1) * 16) = intx4{w0, it, i, sh};
                asm volatile("" ::: "memory");
            }
        }
    }
    float s = (float)(rsum.x + rsum.y + rsum.z + rsum.w) + (float)dsum;
    for (int i = 0; i < 8; ++i) for (int q = 0; q < 16; ++q) s += acc[i][q];
    __syncthreads();
    s += reinterpret_cast<const float *>(lds)[t];
    out[blockIdx.x * kThreads + t] = s;
}

template <int MODE, int PAIRS>
double run(float *out, int iters)     // nanoseconds per iteration
{
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    hipLaunchKernelGGL((cost_kernel<MODE, PAIRS>), dim3(kBlocks), dim3(kThreads), 0, 0, out, 200, 1);
    CK(hipDeviceSynchronize());
    CK(hipEventRecord(e0));
    hipLaunchKernelGGL((cost_kernel<MODE, PAIRS>), dim3(kBlocks), dim3(kThreads), 0, 0, out, iters, 1);
    CK(hipEventRecord(e1));
    CK(hipEventSynchronize(e1));
    float ms;
    CK(hipEventElapsedTime(&ms, e0, e1));
    return ms * 1e6 / iters;
}

// The 16 x 16 x 32 form of the bf16 MFMA (half the flop per instruction, the same peak rate): RND 0 constant, 1
// pseudo-random operands; HALFPAIRS BFP16 decode pairs per TWO MFMAs (i.e. per 32768 flop, the unit of cost_kernel),
// issued after the second MFMA of each pair.
template <int RND, int HALFPAIRS>
__global__ void __launch_bounds__(kThreads) cost16_kernel(float *out, int iters, int seed)
{
    const int t = threadIdx.x;
    bf16x8 a, b;
    for (int e = 0; e < 8; ++e) { a[e] = (__bf16)(float)((t + e) % 3); b[e] = (__bf16)(float)((t + e) % 5); }
    if (RND) {
        union { unsigned u[4]; bf16x8 v; } ua, ub;
        unsigned r = t * 2654435761u + 12345u;
        for (int e = 0; e < 4; ++e) {
            r = r * 1664525u + 1013904223u; ua.u[e] = (r & 0x807F807Fu) | 0x3C003C00u | ((r >> 3) & 0x03800380u);
            r = r * 1664525u + 1013904223u; ub.u[e] = (r & 0x807F807Fu) | 0x3C003C00u | ((r >> 3) & 0x03800380u);
        }
        a = ua.v; b = ub.v;
    }
    floatx4 acc[16];
    for (int i = 0; i < 16; ++i) for (int v = 0; v < 4; ++v) acc[i][v] = 0.f;
    int w0 = seed + t, sh = seed & 3;
    unsigned dsum = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[i], 0, 0, 0);
            FENCE();
            if (i & 1) {
#pragma unroll
                for (int v = 0; v < HALFPAIRS; ++v) {
                    const float f0 = ldexpf(byte_to_float(w0, (2 * v) & 3), sh), f1 = ldexpf(byte_to_float(w0, (2 * v + 1) & 3), sh);
                    union { bf16x2 p; unsigned u; } pk;
                    pk.p = bf16x2{(__bf16)f0, (__bf16)f1};
                    dsum ^= pk.u;
                    w0 += 0x01010101;
                }
            }
            FENCE();
        }
    }
    float s = (float)dsum;
    for (int i = 0; i < 16; ++i) for (int q = 0; q < 4; ++q) s += acc[i][q];
    out[blockIdx.x * kThreads + t] = s;
}

template <int RND, int HALFPAIRS>
double run16(float *out, int iters)     // nanoseconds per iteration
{
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    hipLaunchKernelGGL((cost16_kernel<RND, HALFPAIRS>), dim3(kBlocks), dim3(kThreads), 0, 0, out, 200, 1);
    CK(hipDeviceSynchronize());
    CK(hipEventRecord(e0));
    hipLaunchKernelGGL((cost16_kernel<RND, HALFPAIRS>), dim3(kBlocks), dim3(kThreads), 0, 0, out, iters, 1);
    CK(hipEventRecord(e1));
    CK(hipEventSynchronize(e1));
    float ms;
    CK(hipEventElapsedTime(&ms, e0, e1));
    return ms * 1e6 / iters;
}


__device__ __forceinline__ unsigned rnd_bf16x2(unsigned &r) { r = r * 1664525u + 1013904223u; return (r & 0x807F807Fu) | 0x3C003C00u | ((r >> 3) & 0x03800380u); }

// The GEMM kernel's on-CU instruction mix on pseudo-random operands, built up step by step, with no global
// memory traffic and no barriers: what the power limit leaves of the matrix pipes' throughput once the
// fragment reads, the decode and the staging stores run next to them.  F is a set of flags:
// 1: the MFMA operands rotate over 4 register sets (they change from one MFMA to the next, as in the GEMM);
// 2: the operands come from LDS, one b128 A fragment and one transposing b64 B half-fragment per 2 MFMAs
//    (the GEMM's 2 x 4 wave grid: 16 + 16 reads per 32 MFMAs);
// 4: waves 0-3 decode one BFP16 pair per MFMA (half a pair per MFMA over the SIMD's two waves);
// 8: waves 0-3 store 16 decoded bytes per lane to LDS every 8 MFMAs.
template <int F>
__global__ void __launch_bounds__(kThreads) mix_kernel(float *out, int iters, int seed)
{
    __shared__ __attribute__((aligned(16))) char lds[kLds];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    unsigned r = t * 2654435761u + 12345u + blockIdx.x;
    for (int i = t; i < kLds / 4; i += kThreads) reinterpret_cast<unsigned *>(lds)[i] = rnd_bf16x2(r);
    __syncthreads();
    bf16x8 a[4], b[4];
    for (int s = 0; s < 4; ++s) {
        union { unsigned u[4]; bf16x8 v; } ua, ub;
        for (int e = 0; e < 4; ++e) { ua.u[e] = rnd_bf16x2(r); ub.u[e] = rnd_bf16x2(r); }
        a[s] = ua.v; b[s] = ub.v;
    }
    floatx16 acc[8];
    for (int i = 0; i < 8; ++i) for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    int w0 = seed + t, sh = seed & 3;
    unsigned dsum = 0;
    const char *frag = lds + (wave & 3) * 4608 + (lane & 31) * 144 + (lane >> 5) * 16;
    const int blk = lane >> 4, j = lane & 15, rr = j >> 2;
    const char *tr = lds + 24576 + (8 * (blk >> 1) + rr) * 512 + (((4 * (wave & 3) + 2 * (blk & 1) + ((j & 3) >> 1)) ^ (rr << 2)) * 16) + (j & 1) * 8;
    char *wr = lds + 36864 + (t >> 2) * 144 + (t & 3) * 32;
    typedef __attribute__((address_space(3))) shortx4 lds_shortx4;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int s = (F & 1) ? (i & 3) : 0;
            acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[(F & 1) ? ((i >> 1) & 3) : 0], a[s], acc[i], 0, 0, 0);
            FENCE();
            if (F & 2) {
                if ((i & 1) == 0)      // one A fragment per 2 MFMAs, replacing the set used two MFMAs ago
                    a[(i + 2) & 3] = *reinterpret_cast<const bf16x8 *>(frag + ((it + i) & 3) * 32);
                else {                  // one B half-fragment (tr_b64) per 2 MFMAs
                    union { shortx4 s[2]; bf16x8 v; } u; u.v = b[((i >> 1) + 2) & 3];
                    u.s[(i >> 1) & 1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_shortx4 *)(tr + ((it + i) & 1) * 2048 + ((i >> 1) & 1) * 256));
                    b[((i >> 1) + 2) & 3] = u.v;
                }
            }
            if ((F & 4) && wave < 4) {
                const float f0 = ldexpf(byte_to_float(w0, (2 * i) & 3), sh), f1 = ldexpf(byte_to_float(w0, (2 * i + 1) & 3), sh);
                union { bf16x2 p; unsigned u; } pk;
                pk.p = bf16x2{(__bf16)f0, (__bf16)f1};
                dsum ^= pk.u;
                w0 += 0x01010101;
            }
            if ((F & 8) && wave < 4 && i == 7) {
                *reinterpret_cast<intx4 *>(wr + (it & 1) * 16) = intx4{(int)dsum, w0, (int)dsum ^ w0, it};
            }
            FENCE();
        }
    }
    float s = (float)dsum;
    for (int i = 0; i < 8; ++i) for (int q = 0; q < 16; ++q) s += acc[i][q];
    __syncthreads();
    s += reinterpret_cast<const float *>(lds)[t];
    out[blockIdx.x * kThreads + t] = s;
}

template <int F>
void run_mix(float *out, int iters, const char *what)
{
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    hipLaunchKernelGGL((mix_kernel<F>), dim3(kBlocks), dim3(kThreads), 0, 0, out, 2000, 1);
    CK(hipDeviceSynchronize());
    CK(hipEventRecord(e0));
    hipLaunchKernelGGL((mix_kernel<F>), dim3(kBlocks), dim3(kThreads), 0, 0, out, iters, 1);
    CK(hipEventRecord(e1));
    CK(hipEventSynchronize(e1));
    float ms;
    CK(hipEventElapsedTime(&ms, e0, e1));
    const double x = ms * 1e6 / iters / 16.0;
    printf("mix_kernel<%2d>   %-62s %6.2f ns per MFMA per SIMD = %.0f TFLOP/s\n", F, what, x, 32768.0 * 1024 / x / 1e3);
}

// Issue cost of single VALU instructions next to MFMAs: every wave (two per SIMD) issues one MFMA and then N copies
// of one instruction per slot; the difference between N = 16 and N = 8 is what 8 instructions cost.
template <int KIND> __device__ __forceinline__ void one_op(unsigned &x, unsigned y, float &f, float g)
{
    if (KIND == 0) asm volatile("v_add_u32_e32 %0, %1, %0" : "+v"(x) : "v"(y));
    if (KIND == 1) asm volatile("v_cvt_f32_i32_sdwa %0, sext(%1) dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_1" : "=v"(f) : "v"(y));
    if (KIND == 2) asm volatile("v_cvt_f32_ubyte1_e32 %0, %1" : "=v"(f) : "v"(y));
    if (KIND == 3) asm volatile("v_ldexp_f32 %0, %1, %2" : "=v"(f) : "v"(g), "v"(y));
    if (KIND == 4) asm volatile("v_mul_f32_e32 %0, %1, %0" : "+v"(f) : "v"(g));
    if (KIND == 5) asm volatile("v_fma_f32 %0, %1, %2, %2" : "=v"(f) : "v"(g), "v"(g));
    if (KIND == 6) asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(x) : "v"(f), "v"(g));
    if (KIND == 7) asm volatile("v_perm_b32 %0, %1, %2, %3" : "=v"(x) : "v"(y), "v"(x), "v"(y));
    if (KIND == 8) asm volatile("v_pk_add_u16 %0, %1, %0" : "+v"(x) : "v"(y));
    if (KIND == 9) asm volatile("v_bfe_u32 %0, %1, 8, 8" : "=v"(x) : "v"(y));
}

template <int KIND, int N>
__global__ void __launch_bounds__(kThreads) op_kernel(float *out, int iters, int seed)
{
    bf16x8 a, b;
    for (int t = 0; t < 8; ++t) { a[t] = (__bf16)(float)(threadIdx.x % 3); b[t] = (__bf16)(float)(threadIdx.x % 5); }
    floatx16 acc[8];
    for (int i = 0; i < 8; ++i) for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    unsigned x[4] = {1u + seed, 2u, 3u, 4u};
    float f[4] = {1.f, 2.f, 3.f, 4.f};
    unsigned y = seed + threadIdx.x;
    float g = 1.5f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
            FENCE();
#pragma unroll
            for (int v = 0; v < N; ++v) one_op<KIND>(x[v & 3], y, f[v & 3], g);
            FENCE();
        }
    }
    float s = 0;
    for (int i = 0; i < 8; ++i) for (int q = 0; q < 16; ++q) s += acc[i][q];
    out[blockIdx.x * kThreads + threadIdx.x] = s + x[0] + x[1] + x[2] + x[3] + f[0] + f[1] + f[2] + f[3];
}

template <int KIND, int N>
double run_op(float *out)     // nanoseconds per MFMA per SIMD
{
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    const int iters = 4000;
    hipLaunchKernelGGL((op_kernel<KIND, N>), dim3(kBlocks), dim3(kThreads), 0, 0, out, 10, 1);
    CK(hipDeviceSynchronize());
    CK(hipEventRecord(e0));
    hipLaunchKernelGGL((op_kernel<KIND, N>), dim3(kBlocks), dim3(kThreads), 0, 0, out, iters, 1);
    CK(hipEventRecord(e1));
    CK(hipEventSynchronize(e1));
    float ms;
    CK(hipEventElapsedTime(&ms, e0, e1));
    return ms * 1e6 / (iters * 16.0);
}

template <int KIND>
void op_cost(float *out, const char *name)
{
    const double a = run_op<KIND, 8>(out), b = run_op<KIND, 16>(out);
    printf("op_kernel  %-26s  MFMA + 8: %6.2f ns   MFMA + 16: %6.2f ns   => %.2f ns per instruction, %.1f ns for the MFMA alone\n",
           name, a, b, (b - a) / 8.0, a - (b - a));
}

int main()
{
    float *out;
    CK(hipMalloc(&out, kBlocks * kThreads * sizeof(float)));
    const int iters = 20000;
    printf("every experiment: %d workgroups x %d threads, %d iterations (after a 200-iteration warm-up launch of the same kernel)\n", kBlocks, kThreads, iters);
    double c[4];
    // an iteration issues 8 MFMAs per wave, 16 per SIMD (two waves)
    c[0] = run<0, 0>(out, iters) / 16.0; printf("cost_kernel<0,0>  MFMA 32x32x16 bf16, 0 decode pairs per MFMA: %6.2f ns per MFMA per SIMD\n", c[0]);
    c[1] = run<0, 1>(out, iters) / 16.0; printf("cost_kernel<0,1>  MFMA 32x32x16 bf16, 1 decode pair  per MFMA: %6.2f ns per MFMA per SIMD\n", c[1]);
    c[2] = run<0, 2>(out, iters) / 16.0; printf("cost_kernel<0,2>  MFMA 32x32x16 bf16, 2 decode pairs per MFMA: %6.2f ns per MFMA per SIMD\n", c[2]);
    c[3] = run<0, 3>(out, iters) / 16.0; printf("cost_kernel<0,3>  MFMA 32x32x16 bf16, 3 decode pairs per MFMA: %6.2f ns per MFMA per SIMD\n", c[3]);
    // LDS: 8 waves x 8 instructions per iteration per CU
    double x = run<1, 0>(out, iters) / 64.0; printf("cost_kernel<1,0>  ds_read_b128 (A fragment pattern):       %5.2f ns per wave instruction per CU, %6.1f B/ns\n", x, 1024.0 / x);
    x = run<2, 0>(out, iters) / 64.0;        printf("cost_kernel<2,0>  ds_read_b64_tr_b16 (B fragment pattern): %5.2f ns per wave instruction per CU, %6.1f B/ns\n", x, 512.0 / x);
    x = run<3, 0>(out, iters) / 64.0;        printf("cost_kernel<3,0>  ds_write_b128 (A staging pattern):       %5.2f ns per wave instruction per CU, %6.1f B/ns\n", x, 1024.0 / x);
    // power: long runs (0.1 - 0.2 s, the chip's power management needs that long to settle), constants vs random operands
    x = run<0, 0>(out, 1000000) / 16.0; printf("cost_kernel<0,0>  MFMA only, constant operands, 1e6 iterations: %6.2f ns per MFMA per SIMD = %.0f TFLOP/s\n", x, 32768.0 * 1024 / x / 1e3);
    x = run<4, 0>(out, 1000000) / 16.0; printf("cost_kernel<4,0>  MFMA only, random operands,   1e6 iterations: %6.2f ns per MFMA per SIMD = %.0f TFLOP/s\n", x, 32768.0 * 1024 / x / 1e3);
    x = run<4, 1>(out, 1000000) / 16.0; printf("cost_kernel<4,1>  random operands + 1 decode pair per MFMA:     %6.2f ns per MFMA per SIMD = %.0f TFLOP/s\n", x, 32768.0 * 1024 / x / 1e3);
    // the GEMM's instruction mix on random operands, 7e5 iterations each (0.2 - 0.3 s)
    run_mix<1>(out, 700000, "MFMA only, operands rotate over 4 register sets");
    run_mix<3>(out, 700000, "+ operands from LDS (0.5 b128 + 0.5 tr_b64 per MFMA)");
    run_mix<7>(out, 700000, "+ half a BFP16 decode pair per MFMA (waves 0-3)");
    run_mix<15>(out, 700000, "+ LDS stores of the decoded A (waves 0-3)");
    run_mix<5>(out, 700000, "register operands + the decode, no LDS");
    // single VALU instructions next to MFMAs (constant operands: the clock stays near its maximum)
    op_cost<0>(out, "v_add_u32");
    op_cost<1>(out, "v_cvt_f32_i32 (byte select)");
    op_cost<2>(out, "v_cvt_f32_ubyte1");
    op_cost<3>(out, "v_ldexp_f32");
    op_cost<4>(out, "v_mul_f32");
    op_cost<5>(out, "v_fma_f32");
    op_cost<6>(out, "v_cvt_pk_bf16_f32");
    op_cost<7>(out, "v_perm_b32");
    op_cost<8>(out, "v_pk_add_u16");
    op_cost<9>(out, "v_bfe_u32");
    // the 16 x 16 x 32 form: an iteration issues 16 MFMAs per wave = 32 per SIMD = 16 units of 32768 flop per SIMD
    double d[4];
    d[0] = run16<0, 0>(out, iters) / 16.0; printf("cost16_kernel<0,0> MFMA 16x16x32 bf16, 0 decode pairs per 2 MFMAs: %6.2f ns per 2 MFMAs per SIMD\n", d[0]);
    d[1] = run16<0, 1>(out, iters) / 16.0; printf("cost16_kernel<0,1> MFMA 16x16x32 bf16, 1 decode pair  per 2 MFMAs: %6.2f ns per 2 MFMAs per SIMD\n", d[1]);
    d[2] = run16<0, 2>(out, iters) / 16.0; printf("cost16_kernel<0,2> MFMA 16x16x32 bf16, 2 decode pairs per 2 MFMAs: %6.2f ns per 2 MFMAs per SIMD\n", d[2]);
    d[3] = run16<0, 3>(out, iters) / 16.0; printf("cost16_kernel<0,3> MFMA 16x16x32 bf16, 3 decode pairs per 2 MFMAs: %6.2f ns per 2 MFMAs per SIMD\n", d[3]);
    x = run16<0, 0>(out, 1000000) / 16.0; printf("cost16_kernel<0,0> MFMA only, constant operands, 1e6 iterations: %6.2f ns per 2 MFMAs per SIMD = %.0f TFLOP/s\n", x, 32768.0 * 1024 / x / 1e3);
    x = run16<1, 0>(out, 1000000) / 16.0; printf("cost16_kernel<1,0> MFMA only, random operands,   1e6 iterations: %6.2f ns per 2 MFMAs per SIMD = %.0f TFLOP/s\n", x, 32768.0 * 1024 / x / 1e3);
    x = run16<1, 1>(out, 1000000) / 16.0; printf("cost16_kernel<1,1> random operands + 1 decode pair per 2 MFMAs:  %6.2f ns per 2 MFMAs per SIMD = %.0f TFLOP/s\n", x, 32768.0 * 1024 / x / 1e3);
    x = run<4, 0>(out, 1000000) / 16.0; printf("cost_kernel<4,0>  32x32x16 again, random operands, 1e6 iterations: %6.2f ns per MFMA per SIMD = %.0f TFLOP/s\n", x, 32768.0 * 1024 / x / 1e3);
    return 0;
}
