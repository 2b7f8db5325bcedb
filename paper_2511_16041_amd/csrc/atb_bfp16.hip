// BFP16 quantiser and stand-alone decoder for gfx950.
//
// BFP16 (Sec. 2.4 of arXiv 2511.16041): 8 consecutive values along K share one
// 8-bit exponent, each keeps an 8-bit mantissa.  The reading implemented here:
//   E = max over the block of the fp32 biased exponent field (= 127 + floor(log2|x|)
//       for normal x; fp32 subnormals and zeros contribute 0),
//   m = clamp(round_to_nearest_even(x * 2^(133 - E)), -127, 127),
//   value = m * 2^(E - 133).
// Both kernels are HBM-bound streaming kernels.  The BFP16
// buffer is K-panel-major (see include/atb.h): [panel of 64 k][row][64] mantissas, [panel][row][8] exponents.
#include "atb_internal.h"

namespace atb {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ unsigned exp_field(float x) { return (__float_as_uint(x) >> 23) & 0xFFu; }

// Quantiser.  A wave covers 16 rows x 128 k (two panels of the K-panel-major output); the 4 waves of a
// workgroup sit side by side along k.  In step v lanes 0-31 take row 2v and lanes 32-63 row 2v + 1, four
// consecutive k each, so a load instruction reads two contiguous runs of 512 B and the mantissa store of the
// same step writes, per panel, the 2 x 64 B of the row pair, which are one 128-byte line of the output.  A
// BFP16 block is the 8 values of two neighbouring lanes, which exchange their exponent maxima.  The 16 x 16
// exponent bytes of the wave are collected in LDS and leave as two contiguous runs of 128 B.  Chunks beyond K
// (the tail of the last panel) are written as zero.
__global__ void __launch_bounds__(256) quantize_kernel(const float *__restrict__ A, int64_t lda,
                                                       int8_t *__restrict__ Am, uint8_t *__restrict__ Ae,
                                                       int64_t M, int64_t K, int64_t panels, int64_t kblocks)
{
    __shared__ __attribute__((aligned(8))) uint8_t exps[4][2][16][8];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, half = lane >> 5, q = lane & 31;
    const int64_t r0 = ((int64_t)blockIdx.x / kblocks) * 16;
    const int64_t kg = ((int64_t)blockIdx.x % kblocks) * 4 + wave;       // group of 128 k
    const int64_t k = kg * 128 + 4 * q;
    const int64_t panel = kg * 2 + (q >> 4);
    const int kin = 4 * (q & 15);
#pragma unroll
    for (int v = 0; v < 8; ++v) {
        const int64_t row = r0 + 2 * v + half;
        // the input is read once: non-temporal loads (+12 % whether or not the input was in a cache before the
        // launch); the output keeps ordinary stores, its reader comes next
        floatx4 f = {0.0f, 0.0f, 0.0f, 0.0f};
        if (row < M && k < K) f = __builtin_nontemporal_load(reinterpret_cast<const floatx4 *>(A + row * lda + k));     // K % 8 == 0: k < K implies k + 4 <= K
        unsigned e = max(max(exp_field(f.x), exp_field(f.y)), max(exp_field(f.z), exp_field(f.w)));
        e = max(e, (unsigned)__shfl_xor((int)e, 1));
        const int shift = 133 - (int)e;
        const float x[4] = {f.x, f.y, f.z, f.w};
        unsigned w = 0;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            float r = rintf(ldexpf(x[t], shift));           // exact power-of-two scaling, then RNE
            r = fminf(fmaxf(r, -127.0f), 127.0f);
            w |= ((unsigned)((int)r) & 0xFFu) << (8 * t);
        }
        if (row < M && panel < panels) *reinterpret_cast<unsigned *>(Am + (panel * M + row) * kPanelK + kin) = w;
        if ((q & 1) == 0) exps[wave][q >> 4][2 * v + half][(q & 15) >> 1] = (uint8_t)e;
    }
    __syncthreads();
    if (lane < 32) {
        const int pl = lane >> 4, rl = lane & 15;
        const int64_t row = r0 + rl, pn = kg * 2 + pl;
        if (row < M && pn < panels)
            *reinterpret_cast<uint2 *>(Ae + (pn * M + row) * (kPanelK / 8)) = *reinterpret_cast<const uint2 *>(&exps[wave][pl][rl][0]);
    }
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
    if (M == 0 || panels == 0) return hipSuccess;
    const int64_t kblocks = (panels + 7) / 8;            // a workgroup covers 16 rows x 512 k = 8 panels
    const int64_t blocks = ((M + 15) / 16) * kblocks;
    hipLaunchKernelGGL(quantize_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, A, lda, Am, Ae, M, K, panels, kblocks);
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
