/*
 * CPU oracle for the BFP16 x BF16 GEMM of "Can Asymmetric Tile Buffering Be
 * Beneficial?" (arXiv 2511.16041).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It shares no code, header, table or helper
 * with the HIP path, and nothing in the product path may call it.
 *
 * What it defines (paper passages in brackets):
 *   - BFP16: blocks of 8 values along the reduction dimension share one 8-bit
 *     exponent, each value keeps an 8-bit mantissa [Sec. 2.4 "BFP16 Data Type"].
 *     The paper fixes only "8 values, one 8-bit exponent, 8-bit mantissas";
 *     the reading used here (stated, not printed, by the paper):
 *       shared exponent  e = max over non-zero elements of floor(log2|x|)
 *       stored exponent  E = clamp(e + 127, 0, 254)        (bias of fp32/bf16)
 *       mantissa         m = clamp(RNE(x * 2^(133 - E)), -127, +127)
 *       value            a = m * 2^(E - 133)
 *     so the largest element of a block has 64 <= |x * 2^(133-E)| < 128, a
 *     round-up to 128 saturates to 127 and never bumps the exponent, and an
 *     all-zero block stores E = 0, m = 0.
 *   - GEMM C = A x B with A in R^{MxK}, B in R^{KxN} [Sec. 1], A decoded from
 *     BFP16, B bf16, one fp64 accumulator per output element, k ascending,
 *     then ONE rounding fp64 -> bf16 (round to nearest even).  The tiling of
 *     Sec. 3 (T_MA, T_MC, T_K, T_N) changes data movement, not arithmetic, so
 *     the oracle is this definition; atb_oracle_gemm_tiled walks the ATB loop
 *     nest of Sec. 3 / Sec. 5 ("rho * K/T_K switches per output tile") only to
 *     show that the nest visits every k of every element in ascending order.
 *   - T[i][j] = sum_k |a_ik| |b_kj|, the scale of the acceptance bound
 *     |C_gpu - C_ref| <= 2^-7 * T + 1e-6.
 *
 * Parity unpinned: the paper prints no matrix values and no error metric for
 * its GEMM, so nothing here is checked against numbers from the paper's
 * hardware; the pins are mathematical (tests/test_oracle_*.py).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ bf16 */

/* bf16 = sign(1) exponent(8, bias 127) fraction(7): the top half of an fp32. */
double atb_oracle_bf16_to_double(uint16_t h)
{
    uint32_t w = (uint32_t)h << 16;
    float f;
    memcpy(&f, &w, sizeof f);
    return (double)f;
}

/* Round an fp64 value to bf16, round-to-nearest-even, in ONE rounding (never
 * through fp32).  Overflow goes to infinity, underflow through bf16
 * subnormals (quantum 2^-133) to zero.  Relies on the default FE_TONEAREST
 * mode for rint(). */
uint16_t atb_oracle_bf16_from_double(double x)
{
    uint16_t sign = signbit(x) ? 0x8000u : 0u;
    if (isnan(x)) return (uint16_t)(sign | 0x7FC0u);
    double ax = fabs(x);
    if (ax == 0.0) return sign;
    if (isinf(ax)) return (uint16_t)(sign | 0x7F80u);

    int e2;
    (void)frexp(ax, &e2);           /* ax = f * 2^e2, f in [0.5, 1) */
    int lead = e2 - 1;              /* floor(log2 ax) */
    /* quantum (one unit in the last place) of the bf16 binade that holds ax */
    int q = (lead < -126) ? -133 : lead - 7;
    double scaled = ldexp(ax, -q);  /* exact: power-of-two scaling */
    double r = rint(scaled);        /* ties to even */
    if (lead < -126) {
        /* subnormal range: r in [0, 128]; r == 128 is the smallest normal */
        return (uint16_t)(sign | (uint16_t)r);
    }
    int E = lead + 127;             /* r in [128, 256] */
    if (r >= 256.0) { r = 128.0; E += 1; }
    if (E >= 255) return (uint16_t)(sign | 0x7F80u);
    return (uint16_t)(sign | (uint16_t)(E << 7) | (uint16_t)((int)r - 128));
}

void atb_oracle_bf16_from_double_array(const double *x, int64_t n, uint16_t *out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = atb_oracle_bf16_from_double(x[i]);
}

/* ----------------------------------------------------------------- BFP16 */

/* Quantise fp32 A (M rows, K columns, row pitch lda elements) along K in
 * blocks of 8.  mant is M x K (pitch K), expo is M x K/8 (pitch K/8).
 * Returns 0, or -1 on a bad argument, or the number of non-finite inputs
 * (which are outside the contract; their blocks are left zero). */
int64_t atb_oracle_bfp16_quantize(const float *A, int64_t M, int64_t K, int64_t lda,
                                  int8_t *mant, uint8_t *expo)
{
    if (!A || !mant || !expo || M < 0 || K < 0 || (K % 8) != 0 || lda < K) return -1;
    int64_t bad = 0;
    const int64_t KB = K / 8;
    for (int64_t i = 0; i < M; ++i) {
        for (int64_t kb = 0; kb < KB; ++kb) {
            const float *x = A + i * lda + kb * 8;
            int8_t *m = mant + i * K + kb * 8;
            int have = 0, finite = 1, e = 0;
            for (int t = 0; t < 8; ++t) {
                if (!isfinite(x[t])) { finite = 0; break; }
                if (x[t] != 0.0f) {
                    int e2;
                    (void)frexpf(x[t], &e2);        /* |x| = f * 2^e2, f in [0.5,1) */
                    int fl = e2 - 1;                /* floor(log2 |x|) */
                    if (!have || fl > e) e = fl;
                    have = 1;
                }
            }
            if (!finite) { bad++; have = 0; }
            if (!have) {
                expo[i * KB + kb] = 0;
                for (int t = 0; t < 8; ++t) m[t] = 0;
                continue;
            }
            int E = e + 127;
            if (E < 0) E = 0;
            if (E > 254) E = 254;
            expo[i * KB + kb] = (uint8_t)E;
            for (int t = 0; t < 8; ++t) {
                double r = rint(ldexp((double)x[t], 133 - E));   /* exact scale, RNE */
                if (r > 127.0) r = 127.0;
                if (r < -127.0) r = -127.0;
                m[t] = (int8_t)r;
            }
        }
    }
    return bad;
}

/* a[i][k] = mant[i][k] * 2^(expo[i][k/8] - 133), exactly. */
int atb_oracle_bfp16_decode(const int8_t *mant, const uint8_t *expo, int64_t M, int64_t K,
                            double *out)
{
    if (!mant || !expo || !out || M < 0 || K < 0 || (K % 8) != 0) return -1;
    const int64_t KB = K / 8;
    for (int64_t i = 0; i < M; ++i)
        for (int64_t k = 0; k < K; ++k)
            out[i * K + k] = ldexp((double)mant[i * K + k], (int)expo[i * KB + k / 8] - 133);
    return 0;
}

/* ------------------------------------------------------------------ GEMM */

/* One output row i: acc[j] = sum_k a_ik * b_kj, k ascending, fp64. */
static void gemm_row(const int8_t *mant, const uint8_t *expo, const uint16_t *B,
                     int64_t i, int64_t N, int64_t K,
                     double *acc, double *tacc)
{
    const int64_t KB = K / 8;
    for (int64_t j = 0; j < N; ++j) { acc[j] = 0.0; tacc[j] = 0.0; }
    for (int64_t k = 0; k < K; ++k) {
        double a = ldexp((double)mant[i * K + k], (int)expo[i * KB + k / 8] - 133);
        double aa = fabs(a);
        const uint16_t *brow = B + k * N;
        for (int64_t j = 0; j < N; ++j) {
            double b = atb_oracle_bf16_to_double(brow[j]);
            acc[j] += a * b;
            tacc[j] += aa * fabs(b);
        }
    }
}

/* C_ref for the rows listed in rows[0..nrows) (rows == NULL: rows 0..nrows-1).
 * Outputs are nrows x N, row r of the output belongs to rows[r].
 * C (bf16 bits), S (the fp64 sum before rounding) and T (sum of |a||b|) may
 * each be NULL.  Returns the number of threads used, or -1 on bad arguments. */
int atb_oracle_gemm_rows(const int8_t *mant, const uint8_t *expo, const uint16_t *B,
                         int64_t M, int64_t N, int64_t K,
                         const int64_t *rows, int64_t nrows,
                         uint16_t *C, double *S, double *T)
{
    if (!mant || !expo || !B || M < 0 || N < 0 || K < 0 || (K % 8) != 0 || nrows < 0) return -1;
    for (int64_t r = 0; r < nrows; ++r) {
        int64_t i = rows ? rows[r] : r;
        if (i < 0 || i >= M) return -1;
    }
    int threads = 1;
#ifdef _OPENMP
#pragma omp parallel
#endif
    {
#ifdef _OPENMP
#pragma omp single
        threads = omp_get_num_threads();
#endif
        double *acc = (double *)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1) * 2);
        double *tacc = acc + (N > 0 ? N : 1);
#ifdef _OPENMP
#pragma omp for schedule(dynamic, 1)
#endif
        for (int64_t r = 0; r < nrows; ++r) {
            int64_t i = rows ? rows[r] : r;
            gemm_row(mant, expo, B, i, N, K, acc, tacc);
            for (int64_t j = 0; j < N; ++j) {
                if (C) C[r * N + j] = atb_oracle_bf16_from_double(acc[j]);
                if (S) S[r * N + j] = acc[j];
                if (T) T[r * N + j] = tacc[j];
            }
        }
        free(acc);
    }
    return threads;
}

int atb_oracle_gemm(const int8_t *mant, const uint8_t *expo, const uint16_t *B,
                    int64_t M, int64_t N, int64_t K, uint16_t *C, double *S, double *T)
{
    return atb_oracle_gemm_rows(mant, expo, B, M, N, K, NULL, M, C, S, T);
}

/* The ATB loop nest written out: for every C tile (T_MC x T_N), for every
 * K-step kt, for every A sub-tile s of T_MA rows (rho = T_MC / T_MA of them),
 * one "microkernel" call that adds A_sub(T_MA x T_K) * B_tile(T_K x T_N) into
 * the C tile; the tile is rounded and written once after the last K-step.
 * T_MA == T_MC is symmetric tiling.  Single-threaded, one fp64 accumulator
 * per element of the live C tile.  *switches receives the number of
 * microkernel calls (must equal tiles * rho * ceil(K/T_K)). */
int atb_oracle_gemm_tiled(const int8_t *mant, const uint8_t *expo, const uint16_t *B,
                          int64_t M, int64_t N, int64_t K,
                          int T_MA, int T_MC, int T_K, int T_N,
                          uint16_t *C, int64_t *switches)
{
    if (!mant || !expo || !B || !C || M < 0 || N < 0 || K < 0 || (K % 8) != 0) return -1;
    if (T_MA <= 0 || T_MC <= 0 || T_K <= 0 || T_N <= 0 || (T_MC % T_MA) != 0) return -1;
    const int64_t KB = K / 8;
    const int rho = T_MC / T_MA;
    int64_t calls = 0;
    double *ctile = (double *)malloc(sizeof(double) * (size_t)T_MC * (size_t)T_N);
    if (!ctile) return -1;
    for (int64_t m0 = 0; m0 < M; m0 += T_MC) {
        for (int64_t n0 = 0; n0 < N; n0 += T_N) {
            for (int64_t t = 0; t < (int64_t)T_MC * T_N; ++t) ctile[t] = 0.0;
            for (int64_t k0 = 0; k0 < K; k0 += T_K) {
                for (int s = 0; s < rho; ++s) {
                    ++calls;
                    /* microkernel on A rows [m0 + s*T_MA, +T_MA) */
                    for (int64_t ii = 0; ii < T_MA; ++ii) {
                        int64_t i = m0 + (int64_t)s * T_MA + ii;
                        if (i >= M) break;
                        for (int64_t jj = 0; jj < T_N; ++jj) {
                            int64_t j = n0 + jj;
                            if (j >= N) break;
                            double acc = ctile[((int64_t)s * T_MA + ii) * T_N + jj];
                            for (int64_t k = k0; k < k0 + T_K && k < K; ++k) {
                                double a = ldexp((double)mant[i * K + k],
                                                 (int)expo[i * KB + k / 8] - 133);
                                acc += a * atb_oracle_bf16_to_double(B[k * N + j]);
                            }
                            ctile[((int64_t)s * T_MA + ii) * T_N + jj] = acc;
                        }
                    }
                }
            }
            for (int64_t ii = 0; ii < T_MC && m0 + ii < M; ++ii)
                for (int64_t jj = 0; jj < T_N && n0 + jj < N; ++jj)
                    C[(m0 + ii) * N + (n0 + jj)] =
                        atb_oracle_bf16_from_double(ctile[ii * T_N + jj]);
        }
    }
    free(ctile);
    if (switches) *switches = calls;
    return 0;
}
