// BFP16 quantiser and stand-alone decoder for gfx950.
//
// BFP16 (Sec. 2.4 of arXiv 2511.16041): 8 consecutive values along K share one
// 8-bit exponent, each keeps an 8-bit mantissa.  The reading implemented here:
//   E = max over the block of the fp32 biased exponent field (= 127 + floor(log2|x|)
//       for normal x; fp32 subnormals and zeros contribute 0),
//   m = clamp(round_to_nearest_even(x * 2^(133 - E)), -127, 127),
//   value = m * 2^(E - 133).
// Both kernels are HBM-bound streaming kernels: 16 elements per lane, 16-byte accesses.  The BFP16
// buffer is K-panel-major (see include/atb.h): [panel of 64 k][row][64] mantissas, [panel][row][8] exponents.
#include "atb_internal.h"

namespace atb {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ unsigned exp_field(float x) { return (__float_as_uint(x) >> 23) & 0xFFu; }

// Quantise 8 values that share exponent E; returns the mantissas packed little-endian in two words.
__device__ __forceinline__ void quantize_block(const float (&x)[8], unsigned &E, int &w0, int &w1)
{
    unsigned e = 0;
#pragma unroll
    for (int t = 0; t < 8; ++t) e = max(e, exp_field(x[t]));
    E = e;
    const int shift = 133 - (int)e;
    unsigned b[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        float r = rintf(ldexpf(x[t], shift));           // exact power-of-two scaling, then RNE
        r = fminf(fmaxf(r, -127.0f), 127.0f);
        b[t] = (unsigned)((int)r) & 0xFFu;
    }
    w0 = (int)(b[0] | (b[1] << 8) | (b[2] << 16) | (b[3] << 24));
    w1 = (int)(b[4] | (b[5] << 8) | (b[6] << 16) | (b[7] << 24));
}

// One lane per 16 consecutive k of a row (two BFP16 blocks).  Lanes are numbered (group of 256 k,
// row, chunk within the group): a wave covers 4 rows x 256 k, reads 4 runs of 1 KiB of fp32 and writes,
// per panel of the K-panel-major output, 4 rows x 64 mantissa bytes that are contiguous.  Chunks
// beyond K (the tail of the last panel) are written as zero.
__global__ void __launch_bounds__(256) quantize_kernel(const float *__restrict__ A, int64_t lda,
                                                       int8_t *__restrict__ Am, uint8_t *__restrict__ Ae,
                                                       int64_t M, int64_t K, int64_t panels)
{
    constexpr int CPG = 16;                           // chunks per group of 256 k (4 panels)
    const int64_t groups = (panels * (kPanelK / 16) + CPG - 1) / CPG;
    const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= groups * M * CPG) return;
    const int64_t group = c / (M * CPG), row = (c / CPG) % M;
    const int64_t k0 = (group * CPG + c % CPG) * 16;
    const int64_t panel = k0 / kPanelK, kin = k0 % kPanelK;
    if (panel >= panels) return;
    const float *src = A + row * lda + k0;

    float x[16];
    if (k0 + 16 <= K) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            float4 f = *reinterpret_cast<const float4 *>(src + 4 * v);
            x[4 * v] = f.x; x[4 * v + 1] = f.y; x[4 * v + 2] = f.z; x[4 * v + 3] = f.w;
        }
    } else {
#pragma unroll
        for (int t = 0; t < 16; ++t) x[t] = (k0 + t < K) ? src[t] : 0.0f;
    }
    float lo[8], hi[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) { lo[t] = x[t]; hi[t] = x[8 + t]; }
    unsigned E0, E1;
    int4 m;
    quantize_block(lo, E0, m.x, m.y);
    quantize_block(hi, E1, m.z, m.w);
    *reinterpret_cast<int4 *>(Am + (panel * M + row) * kPanelK + kin) = m;
    *reinterpret_cast<unsigned short *>(Ae + (panel * M + row) * (kPanelK / 8) + (kin >> 3)) = (unsigned short)(E0 | (E1 << 8));
}

__global__ void __launch_bounds__(256) decode_kernel(const int8_t *__restrict__ Am, const uint8_t *__restrict__ Ae,
                                                     uint16_t *__restrict__ out, int64_t M, int64_t K)
{
    const int64_t blocks_per_row = K / 8;
    const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= M * blocks_per_row) return;
    const int64_t row = c / blocks_per_row, kb = c % blocks_per_row;
    const int64_t panel = (kb * 8) / kPanelK, bin = kb % (kPanelK / 8);
    const int2 w = *reinterpret_cast<const int2 *>(Am + (panel * M + row) * kPanelK + bin * 8);
    const int shift = (int)Ae[(panel * M + row) * (kPanelK / 8) + bin] - 133;
    bf16x8 r;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        r[t] = (__bf16)ldexpf((float)(int)(signed char)(w.x >> (8 * t)), shift);
        r[4 + t] = (__bf16)ldexpf((float)(int)(signed char)(w.y >> (8 * t)), shift);
    }
    uint16_t *dst = out + row * K + kb * 8;      // K % 8 == 0: 16-byte aligned when `out` is
    *reinterpret_cast<bf16x8 *>(dst) = r;
}

}  // namespace

hipError_t launch_quantize(const float *A, int64_t lda, int8_t *Am, uint8_t *Ae, int64_t M, int64_t K,
                           hipStream_t stream)
{
    const int64_t panels = (K + kPanelK - 1) / kPanelK;
    const int64_t n = M * ((panels * (kPanelK / 16) + 15) / 16) * 16;
    if (n == 0) return hipSuccess;
    const int64_t blocks = (n + 255) / 256;
    hipLaunchKernelGGL(quantize_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, A, lda, Am, Ae, M, K, panels);
    return hipGetLastError();
}

hipError_t launch_decode(const int8_t *Am, const uint8_t *Ae, uint16_t *out, int64_t M, int64_t K,
                         hipStream_t stream)
{
    const int64_t n = M * (K / 8);
    if (n == 0) return hipSuccess;
    const int64_t blocks = (n + 255) / 256;
    hipLaunchKernelGGL(decode_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, Am, Ae, out, M, K);
    return hipGetLastError();
}

}  // namespace atb
