// Host program for the sanitizer build (tests/test_host_sanitizers.py): walks the argument paths of the
// C ABI, the model and the selector, and runs the C oracle on small heap buffers of exactly the documented
// sizes, so that AddressSanitizer sees any access past them and UBSan any undefined arithmetic.
// Exit status 0 = every expectation held (the sanitizers abort the program themselves).
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "atb.h"

extern "C" {
int64_t atb_oracle_bfp16_quantize(const float *A, int64_t M, int64_t K, int64_t lda, int8_t *mant, uint8_t *expo);
int atb_oracle_bfp16_decode(const int8_t *mant, const uint8_t *expo, int64_t M, int64_t K, double *out);
int atb_oracle_gemm_rows(const int8_t *mant, const uint8_t *expo, const uint16_t *B, int64_t M, int64_t N, int64_t K,
                         const int64_t *rows, int64_t nrows, uint16_t *C, double *S, double *T);
int atb_oracle_gemm_tiled(const int8_t *mant, const uint8_t *expo, const uint16_t *B, int64_t M, int64_t N, int64_t K,
                          int T_MA, int T_MC, int T_K, int T_N, uint16_t *C, int64_t *switches);
uint16_t atb_oracle_bf16_from_double(double x);
double atb_oracle_bf16_to_double(uint16_t h);
void atb_oracle_bf16_from_double_array(const double *x, int64_t n, uint16_t *out);
}

static int failures = 0;
#define EXPECT(cond)                                                                   \
    do {                                                                               \
        if (!(cond)) { std::printf("FAILED line %d: %s\n", __LINE__, #cond); ++failures; } \
    } while (0)

static unsigned lcg(unsigned &s) { s = s * 1664525u + 1013904223u; return s >> 8; }

static void oracle_paths()
{
    const int64_t M = 7, K = 24, N = 9, lda = 29;
    unsigned seed = 7;
    // exact-size heap buffers: an access one element too far is a heap-buffer-overflow
    float *A = (float *)std::malloc(sizeof(float) * ((M - 1) * lda + K));
    for (int64_t i = 0; i < M; ++i)
        for (int64_t k = 0; k < K; ++k)
            A[i * lda + k] = std::ldexp((float)((int)(lcg(seed) % 2001) - 1000), (int)(lcg(seed) % 40) - 30);
    for (int64_t k = 8; k < 16; ++k) A[2 * lda + k] = 0.0f;                              // an all-zero block
    A[3 * lda + 5] = 3.0e38f;                                                             // largest exponents
    A[4 * lda + 1] = 1.0e-44f;                                                            // subnormal fp32
    int8_t *mant = (int8_t *)std::malloc(M * K);
    uint8_t *expo = (uint8_t *)std::malloc(M * K / 8);
    EXPECT(atb_oracle_bfp16_quantize(A, M, K, lda, mant, expo) == 0);
    EXPECT(atb_oracle_bfp16_quantize(A, M, K, K - 1, mant, expo) != 0);                   // lda < K
    EXPECT(atb_oracle_bfp16_quantize(A, M, 12, lda, mant, expo) != 0);                    // K % 8
    A[0] = INFINITY;
    EXPECT(atb_oracle_bfp16_quantize(A, 1, 8, lda, mant, expo) != 0);                     // non-finite input
    A[0] = 1.0f;
    EXPECT(atb_oracle_bfp16_quantize(A, M, K, lda, mant, expo) == 0);
    for (int64_t i = 0; i < M * K; ++i) EXPECT(mant[i] >= -127);
    double *dec = (double *)std::malloc(sizeof(double) * M * K);
    EXPECT(atb_oracle_bfp16_decode(mant, expo, M, K, dec) == 0);
    uint16_t *B = (uint16_t *)std::malloc(sizeof(uint16_t) * K * N);
    for (int64_t i = 0; i < K * N; ++i) B[i] = atb_oracle_bf16_from_double(((int)(lcg(seed) % 513) - 256) / 64.0);
    // keep the huge row out of the GEMM (its sums overflow bf16, which is legal but uninteresting here)
    for (int64_t k = 0; k < K; ++k) mant[3 * K + k] = (int8_t)(k % 5);
    for (int64_t k = 0; k < K / 8; ++k) expo[3 * (K / 8) + k] = 127;
    uint16_t *C = (uint16_t *)std::malloc(sizeof(uint16_t) * M * N);
    double *S = (double *)std::malloc(sizeof(double) * M * N), *T = (double *)std::malloc(sizeof(double) * M * N);
    EXPECT(atb_oracle_gemm_rows(mant, expo, B, M, N, K, nullptr, M, C, S, T) >= 1);
    const int64_t rows[3] = {6, 0, 3};
    uint16_t *C3 = (uint16_t *)std::malloc(sizeof(uint16_t) * 3 * N);
    EXPECT(atb_oracle_gemm_rows(mant, expo, B, M, N, K, rows, 3, C3, nullptr, nullptr) >= 1);
    for (int r = 0; r < 3; ++r) EXPECT(std::memcmp(C3 + r * N, C + rows[r] * N, sizeof(uint16_t) * N) == 0);
    const int64_t bad_rows[1] = {M};
    EXPECT(atb_oracle_gemm_rows(mant, expo, B, M, N, K, bad_rows, 1, C3, nullptr, nullptr) == -1);
    uint16_t *Ct = (uint16_t *)std::malloc(sizeof(uint16_t) * M * N);
    const int tilings[4][4] = {{2, 4, 8, 4}, {3, 3, 16, 5}, {1, 8, 24, 16}, {4, 4, 5, 2}};
    for (const auto &t : tilings) {
        int64_t sw = -1;
        EXPECT(atb_oracle_gemm_tiled(mant, expo, B, M, N, K, t[0], t[1], t[2], t[3], Ct, &sw) == 0);
        EXPECT(std::memcmp(Ct, C, sizeof(uint16_t) * M * N) == 0);                        // tiling changes nothing
        EXPECT(sw == ((M + t[1] - 1) / t[1]) * ((N + t[3] - 1) / t[3]) * (t[1] / t[0]) * ((K + t[2] - 1) / t[2]));
    }
    EXPECT(atb_oracle_gemm_tiled(mant, expo, B, M, N, K, 3, 4, 8, 4, Ct, nullptr) == -1);  // rho not an integer
    const double vals[5] = {0.0, -0.0, 1.0e-45, 3.4e38, -65504.0};
    uint16_t bits[5];
    atb_oracle_bf16_from_double_array(vals, 5, bits);
    EXPECT(bits[0] == 0 && bits[1] == 0x8000);
    EXPECT(atb_oracle_bf16_to_double(0x3F80) == 1.0);
    std::free(A); std::free(mant); std::free(expo); std::free(dec); std::free(B); std::free(C); std::free(S);
    std::free(T); std::free(C3); std::free(Ct);
}

static void api_paths()
{
    for (int s = -1; s <= 8; ++s) EXPECT(atb_status_string((atb_status)s) != nullptr);
    EXPECT(atb_instance_count() == 4);
    int a = 0, b = 0, c = 0, d = 0;
    EXPECT(atb_instance_get(0, &a, &b, &c, &d) == ATB_OK && a == 256 && d == 256);
    EXPECT(atb_instance_get(1, nullptr, nullptr, nullptr, nullptr) == ATB_OK);
    EXPECT(atb_instance_get(-1, &a, &b, &c, &d) == ATB_ERR_INVALID_ARG);
    EXPECT(atb_instance_get(4, &a, &b, &c, &d) == ATB_ERR_INVALID_ARG);
    int rows = 0;
    EXPECT(atb_instance_geometry(3, &a, &b, &c, &rows) == ATB_OK && a == 1 && b == 2 && c == 6 && rows == 32);
    EXPECT(atb_instance_geometry(0, nullptr, nullptr, nullptr, &rows) == ATB_OK && rows == 16);
    EXPECT(atb_instance_geometry(9, &a, &b, &c, &rows) == ATB_ERR_INVALID_ARG);

    atb_bfp16_layout_t lay;
    EXPECT(atb_bfp16_layout(3000, 4104, &lay) == ATB_OK && lay.panels == 65 && lay.man_stride == 3000 * 64);
    EXPECT(lay.exp_off % 256 == 0 && lay.bytes % 256 == 0 && lay.bytes >= lay.exp_off + lay.panels * lay.exp_stride);
    EXPECT(atb_bfp16_layout(0, 8, &lay) == ATB_ERR_INVALID_ARG);
    EXPECT(atb_bfp16_layout(4, 12, &lay) == ATB_ERR_INVALID_ARG);
    EXPECT(atb_bfp16_layout(4, 8, nullptr) == ATB_ERR_INVALID_ARG);
    EXPECT(atb_bfp16_bytes(1, 8) == 512);                                                   // 64 mantissa bytes -> 256, 8 exponent bytes -> 256
    EXPECT(atb_bfp16_bytes(-5, 8) == 0);

    atb_gemm *g = nullptr;
    alignas(16) static char fake[64];
    EXPECT(atb_gemm_create(nullptr, 64, 64, 64, 32, 64, 64, 64) == ATB_ERR_INVALID_ARG);
    EXPECT(atb_gemm_create(&g, 0, 64, 64, 32, 64, 64, 64) == ATB_ERR_INVALID_ARG && g == nullptr);
    EXPECT(atb_gemm_create(&g, 64, 64, 60, 32, 64, 64, 64) == ATB_ERR_INVALID_ARG);
    EXPECT(atb_gemm_create(&g, 64, 64, 64, 0, 64, 64, 64) == ATB_ERR_INVALID_ARG);
    EXPECT(atb_gemm_create(&g, 64, 64, 64, 48, 64, 64, 64) == ATB_ERR_BAD_TILE);
    EXPECT(atb_gemm_create(&g, 64, 64, 64, 64, 64, 64, 64) == ATB_ERR_BAD_TILE);          // legal factors, not in the table
    EXPECT(atb_gemm_create(&g, 64, 64, 64, 256, 256, 64, 512) == ATB_ERR_REG_BUDGET);
    EXPECT(atb_gemm_create(&g, 64, 64, 64, 256, 256, 128, 256) == ATB_ERR_LDS_BUDGET);
    EXPECT(atb_gemm_create(&g, (int64_t)1 << 24, 64, 64, 32, 64, 64, 64) == ATB_ERR_INVALID_ARG);
    EXPECT(atb_gemm_create(&g, 1 << 20, 1 << 20, 64, 32, 64, 64, 64) == ATB_ERR_INVALID_ARG);
    EXPECT(atb_gemm_create_fmt(&g, 64, 64, 64, 32, 64, 64, 64, (atb_format)7, ATB_FMT_BF16) == ATB_ERR_INVALID_ARG);
    EXPECT(atb_gemm_create_fmt(&g, 64, 60, 64, 32, 64, 64, 64, ATB_FMT_BF16, ATB_FMT_BFP16) == ATB_ERR_INVALID_ARG);
    EXPECT(atb_gemm_create_fmt(&g, 512, 512, 512, 32, 256, 128, 256, ATB_FMT_BFP16, ATB_FMT_BF16) == ATB_ERR_BAD_TILE);
    EXPECT(atb_gemm_create_fmt(&g, 512, 512, 512, 32, 64, 64, 64, ATB_FMT_BF16_T, ATB_FMT_BF16) == ATB_ERR_BAD_TILE);
    EXPECT(atb_gemm_create_fmt(&g, 512, 512, 512, 128, 256, 64, 256, ATB_FMT_BF16_T, ATB_FMT_BFP16) == ATB_ERR_INVALID_ARG);
    EXPECT(atb_gemm_create_fmt(&g, 512, 512, 512, 128, 256, 64, 256, ATB_FMT_BF16, ATB_FMT_BF16_T) == ATB_ERR_INVALID_ARG);
    EXPECT(atb_gemm_create_fmt(&g, 512, 500, 512, 128, 256, 64, 256, ATB_FMT_BF16_T, ATB_FMT_BF16) == ATB_OK);
    EXPECT(atb_gemm_run(g, fake, fake, fake, nullptr) == ATB_ERR_HIP);
    atb_gemm_destroy(g);

    EXPECT(atb_gemm_create(&g, 3000, 5000, 4104, 256, 256, 64, 256) == ATB_OK && g != nullptr);
    int64_t wg = 0; int th = 0, lds = 0;
    EXPECT(atb_gemm_launch_info(g, &wg, &th, &lds) == ATB_OK && wg == 240 && th == 512 && lds == 139264);
    EXPECT(atb_gemm_launch_info(g, nullptr, nullptr, nullptr) == ATB_OK);
    EXPECT(atb_gemm_launch_info(nullptr, &wg, &th, &lds) == ATB_ERR_INVALID_ARG);
    EXPECT(atb_gemm_run(nullptr, fake, fake, fake, nullptr) == ATB_ERR_INVALID_ARG);
    EXPECT(atb_gemm_run(g, nullptr, fake, fake, nullptr) == ATB_ERR_INVALID_ARG);
    EXPECT(atb_gemm_run(g, fake, fake + 2, fake, nullptr) == ATB_ERR_INVALID_ARG);         // misaligned B
    EXPECT(atb_gemm_run(g, fake, fake, fake, nullptr) == ATB_ERR_HIP && atb_last_hip_error() != 0);   // the stub launch fails
    atb_gemm_destroy(g);
    EXPECT(atb_gemm_create_fmt(&g, 256, 256, 256, 32, 64, 64, 64, ATB_FMT_BFP16, ATB_FMT_BFP16) == ATB_OK);
    EXPECT(atb_gemm_run(g, fake, fake, fake, nullptr) == ATB_ERR_HIP);
    atb_gemm_destroy(g);
    atb_gemm_destroy(nullptr);

    EXPECT(atb_bfp16_quantize(nullptr, 8, fake, 1, 8, nullptr) == ATB_ERR_INVALID_ARG);
    EXPECT(atb_bfp16_quantize((const float *)fake, 6, fake, 1, 8, nullptr) == ATB_ERR_INVALID_ARG);   // lda < K
    EXPECT(atb_bfp16_quantize((const float *)fake, 8, fake, 1, 8, nullptr) == ATB_ERR_HIP);
    EXPECT(atb_bfp16_decode(fake, fake, 1, 8, nullptr) == ATB_ERR_HIP);
    EXPECT(atb_bfp16_decode(fake, nullptr, 1, 8, nullptr) == ATB_ERR_INVALID_ARG);

    double flop = 0;
    EXPECT(atb_mfma_probe(nullptr, nullptr, 1, 1, 1, 16, nullptr, &flop) == ATB_ERR_INVALID_ARG);
    EXPECT(atb_mfma_probe(fake, nullptr, 0, 1, 1, 16, nullptr, &flop) == ATB_ERR_INVALID_ARG);
    EXPECT(atb_mfma_probe(fake, fake + 4, 1, 1, 1, 16, nullptr, &flop) == ATB_ERR_INVALID_ARG);          // clocks misaligned
    EXPECT(atb_mfma_probe(fake, nullptr, 1, 1, 1, 8, nullptr, &flop) == ATB_ERR_INVALID_ARG);                // no such MFMA form
    EXPECT(atb_mfma_probe(fake, nullptr, 2, 3, 1, 32, nullptr, &flop) == ATB_ERR_HIP && flop == 8.0 * 2 * 3 * 32 * 32768.0);
}

static void model_paths()
{
    atb_hw_params x, m;
    atb_hw_params_xdna2(&x);
    atb_hw_params_mi355x(&m);
    atb_hw_params_xdna2(nullptr);
    atb_hw_params_mi355x(nullptr);
    atb_choice ch;
    EXPECT(atb_model_eval(4096, 2048, 4096, 32, 128, 64, 128, &x, &ch) == ATB_OK && ch.rho == 4 && ch.feasible == 1);
    EXPECT(std::fabs(ch.ai - 410.0) < 1.0);                                                // Table 2, 128x64x128 at rho = 4
    EXPECT(atb_model_eval(4096, 2048, 4096, 128, 128, 64, 128, &x, &ch) == ATB_OK && ch.feasible == 0);
    EXPECT(atb_model_eval(8192, 8192, 8192, 256, 256, 64, 256, nullptr, &ch) == ATB_OK && ch.feasible == 1 && ch.pred_flops > 0);
    EXPECT(atb_model_eval(1, 1, 8, 256, 256, 64, 256, nullptr, &ch) == ATB_OK && std::isfinite(ch.pred_flops));
    EXPECT(atb_model_eval(8192, 8192, 8192, 256, 256, 64, 256, nullptr, nullptr) == ATB_ERR_INVALID_ARG);
    EXPECT(atb_model_eval(8192, 8192, 8192, 96, 256, 64, 256, nullptr, &ch) == ATB_ERR_BAD_TILE);
    atb_hw_params bad = m;
    bad.II = 0.0;
    EXPECT(atb_model_eval(64, 64, 64, 32, 64, 64, 64, &bad, &ch) == ATB_ERR_INVALID_ARG);

    std::vector<atb_choice> ranked(8);
    int count = -1;
    EXPECT(atb_select_tiles(8192, 8192, 8192, nullptr, ranked.data(), 8, &count) == ATB_OK && count == 4);
    for (int i = 1; i < count; ++i)
        EXPECT(ranked[i - 1].feasible > ranked[i].feasible ||
               (ranked[i - 1].feasible == ranked[i].feasible && ranked[i - 1].pred_flops >= ranked[i].pred_flops));
    atb_choice *two = (atb_choice *)std::malloc(2 * sizeof(atb_choice));                   // capacity below count
    EXPECT(atb_select_tiles(16, 8192, 8192, &m, two, 2, &count) == ATB_OK && count == 4);
    EXPECT(atb_select_tiles(16, 8192, 8192, &m, two, 2, nullptr) == ATB_OK);
    std::free(two);
    EXPECT(atb_select_tiles(16, 8192, 8192, nullptr, nullptr, 0, &count) == ATB_OK && count == 4);
    EXPECT(atb_select_tiles(16, 8192, 8192, nullptr, nullptr, 2, &count) == ATB_ERR_INVALID_ARG);
    EXPECT(atb_select_tiles(0, 8192, 8192, nullptr, ranked.data(), 8, &count) == ATB_ERR_INVALID_ARG);
    EXPECT(atb_select_tiles(64, 64, 64, &x, ranked.data(), 8, &count) == ATB_OK);

    atb_micro_model mm;
    EXPECT(atb_model_microkernel(256, 256, 64, 256, 2, 4, 1, 16, &mm) == ATB_OK && mm.n_mfma == 256 && mm.mfma_util > 0 && mm.mfma_util <= 1);
    EXPECT(atb_model_microkernel(256, 256, 64, 256, 2, 4, 1, 16, nullptr) == ATB_ERR_INVALID_ARG);
    EXPECT(atb_model_microkernel(256, 256, 64, 256, 2, 4, 1, 8, &mm) == ATB_ERR_INVALID_ARG);
    EXPECT(atb_model_microkernel(96, 256, 64, 256, 2, 4, 1, 16, &mm) == ATB_ERR_BAD_TILE);
    EXPECT(atb_model_microkernel(32, 64, 40, 64, 1, 2, 6, 32, &mm) == ATB_ERR_BAD_TILE);
}

int main()
{
    oracle_paths();
    api_paths();
    model_paths();
    if (failures) { std::printf("%d expectation(s) failed\n", failures); return 1; }
    std::printf("sanitize_host: ok\n");
    return 0;
}
