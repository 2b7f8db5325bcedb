/*
 * libatb -- BFP16 x BF16 GEMM with asymmetric tile buffering (ATB) for AMD
 * MI355X (gfx950), after "Can Asymmetric Tile Buffering Be Beneficial?"
 * (arXiv 2511.16041).
 *
 * C ABI.  Every pointer argument says whether it is HOST or DEVICE memory.
 * The caller owns every buffer; the library allocates host memory only (in
 * atb_gemm_create) and never device memory.  No function throws, aborts or
 * synchronises the device; every function that can fail returns an
 * atb_status.  Streams are hipStream_t values passed as void* (NULL = the
 * default stream).
 *
 * Operation (Sec. 1 and Sec. 3 of the paper):  C = A x B with A in R^{MxK},
 * B in R^{KxN}, C in R^{MxN}.  A is stored in BFP16 (Sec. 2.4: blocks of 8
 * values along K share one 8-bit exponent and keep an 8-bit mantissa each),
 * B and C are bf16, accumulation is fp32.  The kernel is output-stationary
 * (Sec. 3.1): each workgroup owns one T_MC x T_N tile of C for the whole
 * reduction; per K-step of T_K it keeps a T_K x T_N tile of B resident and
 * streams A through in sub-tiles of T_MA <= T_MC rows (rho = T_MC / T_MA
 * "kernel switches" per K-step, Sec. 5).  T_MA == T_MC is symmetric tiling.
 *
 * BFP16 values (the reading of Sec. 2.4 used throughout):
 *     a[i][k] = m[i][k] * 2^(E[i][k/8] - 133),  m int8 in [-127, 127],
 *     E uint8 = 127 + max over the block of floor(log2 |x|)  (0 for a zero block),
 *     m = clamp(round_to_nearest_even(x * 2^(133 - E)), -127, 127).
 *
 * Device layout of an A_bfp buffer for an M x K matrix (atb_bfp16_layout gives
 * the numbers): K is cut into panels of 64; inside a panel the rows follow
 * each other, so the part of a tile that one K-step needs is one contiguous
 * run of bytes (the GEMM fetches it with fully coalesced 16-byte requests).
 *     mantissa plane  int8  [panels][M][64]  at byte 0,
 *                     panels = ceil(K / 64); m[i][k] at (k/64) * M*64 + i*64 + k%64
 *     exponent plane  uint8 [panels][M][8]   at byte exp_off = round_up(panels * M * 64, 256);
 *                     E[i][k/8] at exp_off + (k/64) * M*8 + i*8 + (k%64)/8
 *     total bytes = round_up(exp_off + panels * M * 8, 256)
 *   Mantissa bytes with k >= K (the tail of the last panel) MUST be zero; the
 *   exponent bytes there are ignored.  9 bytes per 8 elements as in the
 *   paper's packed bfp16ebs8, but planar so that all loads are aligned.
 * B: bf16, row-major K x N, leading dimension N.  C: bf16, row-major M x N,
 * leading dimension N.  A_bfp, B and C must be 16-byte aligned.
 */
#ifndef ATB_H
#define ATB_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum atb_status {
    ATB_OK = 0,
    ATB_ERR_INVALID_ARG = 1, /* NULL pointer, non-positive size, K % 8 != 0, misaligned buffer */
    ATB_ERR_BAD_TILE = 2,    /* T_MC % T_MA != 0, or (T_MA,T_MC,T_K,T_N) is not a compiled instance */
    ATB_ERR_LDS_BUDGET = 3,  /* the tile's A and B buffers exceed the 160 KiB LDS of a CU */
    ATB_ERR_REG_BUDGET = 4,  /* the T_MC x T_N fp32 C tile exceeds the accumulator registers */
    ATB_ERR_HIP = 5,         /* a HIP call failed (no device, bad launch); see atb_last_hip_error */
    ATB_ERR_NOMEM = 6        /* host allocation failed */
} atb_status;

/* Static string for a status code. Never NULL. */
const char *atb_status_string(atb_status s);

/* hipError_t value of the most recent failing HIP call on this thread (0 if none). */
int atb_last_hip_error(void);

/* ------------------------------------------------------------------ GEMM */

typedef struct atb_gemm atb_gemm; /* opaque plan, HOST memory */

/* Plan C[M][N] = A_bfp[M][K] x B[K][N] with the tile factors of Sec. 3
 * (T_MA rows of A buffered per sub-tile, T_MC x T_N C tile, T_K reduction
 * step).  Touches no device.  Requirements: M, N, K >= 1, K % 8 == 0,
 * T_MC % T_MA == 0, and the factors must name a compiled instance (see
 * atb_instance_count / atb_instance_get).  M and N need not be multiples of
 * the tile (edge tiles are masked); K need not be a multiple of T_K.
 * Size limits (32-bit element offsets inside the kernel; ATB_ERR_INVALID_ARG
 * beyond them): M, N <= 2^23, K <= 2^24, every operand below 2^31 elements
 * (M * round_up(K, 64), K * N, M * N; also N * round_up(K, 64) and
 * M * round_up(N, 64) for the BFP16 forms of B and C), and
 * 2 * N * (T_K + 1) < 2^31.
 * On success *out is a new plan, else *out = NULL.
 * Environment (read here, both optional): ATB_LOG=1 prints the plan to
 * stderr; ATB_GROUP_M=<tile rows, 1..65536> overrides the height of the
 * patch of C tiles that the workgroups resident on one XCD cover (the
 * order in which tiles are walked, a measurement aid: results are the same
 * for every value). */
atb_status atb_gemm_create(atb_gemm **out, int64_t M, int64_t N, int64_t K,
                           int T_MA, int T_MC, int T_K, int T_N);

/* Launch the planned GEMM on `hip_stream`; returns after the launch (async).
 * A_bfp: DEVICE, layout above, read-only.  B_bf16: DEVICE, K x N bf16,
 * read-only.  C_bf16: DEVICE, M x N bf16, fully overwritten.  Inputs must be
 * finite.  Reports launch-time errors only. */
atb_status atb_gemm_run(const atb_gemm *g, const void *A_bfp, const void *B_bf16,
                        void *C_bf16, void *hip_stream);

void atb_gemm_destroy(atb_gemm *g);

/* Storage formats of the B and C operands (Sec. 6.1 of the paper lists three
 * precision configurations; its Configs 2 and 3 store every operand as BFP16).
 * A is always BFP16; accumulation is always fp32 in the MFMA accumulators. */
typedef enum atb_format {
    ATB_FMT_BF16 = 0,
    ATB_FMT_BFP16 = 1,
    ATB_FMT_BF16_T = 2      /* B only: bf16, handed over transposed (see atb_gemm_create_fmt) */
} atb_format;

/* atb_gemm_create with a storage format per operand.  The plan is run with
 * atb_gemm_run, whose B and C pointers then mean:
 *   b_format BF16 : B, K x N bf16 row-major (as in atb_gemm_create).
 *   b_format BFP16: B^T, N x K, as a BFP16 buffer with the layout
 *                   atb_bfp16_layout(N, K), i.e. blocks of 8 along K (the
 *                   reduction dimension, as the format requires, Sec. 2.4)
 *                   with the K index contiguous; atb_bfp16_quantize of a
 *                   row-major N x K fp32 matrix produces it.
 *   b_format BF16_T: B^T, N x K bf16 row-major (leading dimension K, the K index
 *                   contiguous) -- the layout in which frameworks keep the weight of a
 *                   linear layer.  The kernel then reads its B fragments with plain
 *                   16-byte LDS reads instead of transposing ones (half the LDS read
 *                   instructions for B).  Same values, same summation order, same
 *                   result bits as b_format BF16.  Needs c_format BF16, an instance
 *                   with T_K = 64 and a C tile of at least 128 x 256, and
 *                   2 * T_N * K < 2^31 (else ATB_ERR_BAD_TILE / ATB_ERR_INVALID_ARG).
 *   c_format BF16 : C, M x N bf16 row-major.
 *   c_format BFP16: C as a BFP16 buffer with the layout atb_bfp16_layout(M, N)
 *                   (blocks of 8 along N), quantised from the fp32
 *                   accumulators by the same rule as atb_bfp16_quantize;
 *                   the tail of the last panel (columns N .. 64 * panels - 1) is
 *                   written as zero, so the buffer is a valid operand as it is.
 * c_format BFP16 needs N % 8 == 0 (whole blocks; else ATB_ERR_INVALID_ARG);
 * formats other than (BF16, BF16) need an instance that carries the variants: all but (32, 256, 64, 256) and
 * (32, 256, 128, 256), whose four waves of 256 accumulator registers leave none for a second staging pipeline
 * (else ATB_ERR_BAD_TILE).  All else as atb_gemm_create. */
atb_status atb_gemm_create_fmt(atb_gemm **out, int64_t M, int64_t N, int64_t K,
                               int T_MA, int T_MC, int T_K, int T_N,
                               atb_format b_format, atb_format c_format);

/* Launch geometry of a plan, for benches and tests: number of C tiles the
 * launch walks, rounded up to a multiple of 8 (the grid is persistent: it has
 * min(that, workgroups resident on the chip) workgroups, each looping over its
 * tiles), threads per workgroup, static LDS bytes per workgroup. Any pointer
 * may be NULL. */
atb_status atb_gemm_launch_info(const atb_gemm *g, int64_t *workgroups, int *threads, int *lds_bytes);

/* The compiled (T_MA, T_MC, T_K, T_N) instances. */
int atb_instance_count(void);
atb_status atb_instance_get(int index, int *T_MA, int *T_MC, int *T_K, int *T_N);

/* ----------------------------------------------------------------- BFP16 */

typedef struct atb_bfp16_layout_t {
    int64_t panel_k;     /* K extent of a panel: 64 */
    int64_t panels;      /* ceil(K / 64) */
    int64_t man_stride;  /* bytes between panels of the mantissa plane: M * 64 */
    int64_t exp_stride;  /* bytes between panels of the exponent plane: M * 8 */
    int64_t exp_off;     /* byte offset of the exponent plane */
    int64_t bytes;       /* total size of the buffer */
} atb_bfp16_layout_t;

/* Layout of an A_bfp buffer for an M x K matrix (K % 8 == 0). */
atb_status atb_bfp16_layout(int64_t M, int64_t K, atb_bfp16_layout_t *out);

/* Total bytes of an A_bfp buffer; 0 on invalid arguments. */
size_t atb_bfp16_bytes(int64_t M, int64_t K);

/* Quantise A_f32_dev (DEVICE, fp32, M x K, row pitch lda elements, lda >= K,
 * 16-byte aligned rows: lda % 4 == 0) into A_bfp_dev (DEVICE, layout above,
 * atb_bfp16_bytes(M,K) bytes; padding is written as zero).  Async on
 * hip_stream.  Inputs must be finite.  Bit-exact against the definition
 * in the header comment (Sec. 2.4 reading). */
atb_status atb_bfp16_quantize(const float *A_f32_dev, int64_t lda, void *A_bfp_dev,
                              int64_t M, int64_t K, void *hip_stream);

/* Decode an A_bfp buffer to bf16 (DEVICE, M x K, leading dimension K); exact.
 * For inspection and tests; the GEMM decodes inside its own kernel. */
atb_status atb_bfp16_decode(const void *A_bfp_dev, void *A_bf16_dev, int64_t M, int64_t K,
                            void *hip_stream);

/* ------------------------------------------------- model and tile selector */

/* Machine constants of the paper's performance model (Secs. 3 and 5). */
typedef struct atb_hw_params {
    double peak_core_flops;   /* Perf_core^peak: one core (XDNA2) / one CU (MI355X), flop/s */
    int    n_core;            /* N_core */
    int    array_rows;        /* cores sharing a B tile: L2 tile is array_rows*T_MC x array_cols*T_N (Eq. 2) */
    int    array_cols;
    double bw_offchip;        /* BW_offchip, byte/s */
    double buffer_bytes;      /* S of Eq. (1): L1 (XDNA2) or LDS (MI355X) per core */
    double acc_bytes;         /* MI355X only: accumulator-register bytes per core; 0 = C lives in `buffer_bytes` */
    double clock_hz;
    double delta_cycles;      /* delta: cost of one microkernel switch (Sec. 5) */
    double fill_cycles;       /* MI355X extension, 0 on XDNA2: pipeline-fill cost per K-step that an A sub-tile of
                                 T_MC rows exposes; a sub-tile of T_MC/rho rows exposes fill_cycles/rho (see atb_model_eval) */
    double eta, eps, II;      /* Eff_micro(T_K) = eta T_K / (eps + eta II T_K), Eq. (12) */
    double a_bytes, b_bytes, c_bytes; /* bytes per element of A, B, C moved from off-chip */
    double a_buf_bytes, b_buf_bytes;  /* bytes per element of A, B as buffered (Eq. 1); 0 = same as above */
    int    n_b_buffers;       /* B buffers in Eq. (1): the paper uses 2 */
} atb_hw_params;

/* Fill *hw with the paper's XDNA2 constants (Secs. 2.4, 3.2, 5; precision
 * Config 1 byte costs) or with this library's MI355X constants. */
void atb_hw_params_xdna2(atb_hw_params *hw);
void atb_hw_params_mi355x(atb_hw_params *hw);

typedef struct atb_choice {
    int T_MA, T_MC, T_K, T_N;
    int rho;               /* T_MC / T_MA */
    int feasible;          /* buffer (and accumulator) constraints hold */
    double ai;             /* AI_array, Eq. (2)  [flop/byte] */
    double ai_core;        /* AI_rho, Sec. 3.1 */
    double buffer_bytes;   /* left side of Eq. (1) (C term dropped when acc_bytes > 0) */
    double acc_bytes;      /* 4 * T_MC * T_N when acc_bytes > 0 in hw, else 0 */
    double eff_micro;      /* Eq. (12) */
    double eff_core;       /* Eq. (15) */
    double mem_bound;      /* AI_array * BW_offchip, flop/s */
    double compute_bound;  /* Eff_core * Perf_core^peak * N_core, flop/s */
    double pred_flops;     /* Eq. (11): min of the two */
} atb_choice;

/* Evaluate the model (Eqs. 1, 2, 11, 12, 15) for one set of tile factors.
 * hw == NULL means MI355X.  Pure host arithmetic.  Per output tile and K-step
 * the time is  2 T_MC T_N T_K / (Peak_core Eff_micro) + delta rho + fill / rho  (Eq. 14 plus the
 * fill term; with fill_cycles = 0 this is the paper's Eq. 14 / Eq. 15 exactly). */
atb_status atb_model_eval(int64_t M, int64_t N, int64_t K, int T_MA, int T_MC, int T_K, int T_N,
                          const atb_hw_params *hw, atb_choice *out);

/* Rank the compiled instances for a problem by predicted throughput
 * (infeasible ones last): atb_model_eval's prediction, with the compute bound
 * scaled by the measured full-load factor an instance may carry, rounds of
 * tiles counted in workgroups resident per CU, partly filled rounds credited
 * with the clock the idle CUs leave, and a fixed launch cost.  Writes min(capacity, count) entries to `ranked`
 * (HOST) and the number of instances to *count.  ranked[0] is the pick. */
atb_status atb_select_tiles(int64_t M, int64_t N, int64_t K, const atb_hw_params *hw,
                            atb_choice *ranked, int capacity, int *count);

/* ------------------------------------------------- microkernel issue model */

/* Sec. 4 of the paper models its microkernel on a VLIW core: a prolog bounded
 * by load latency and load-unit throughput (Eq. 4), a steady state whose
 * initiation interval is the larger of the MAC pipeline constraint and the
 * load constraint (Eq. 5), an epilog (Eq. 8), and their sum per kernel call
 * (Eq. 9), overlapped when several accumulation clusters are in flight
 * (Eq. 10).  This is the same decomposition for one gfx950 CU, with unit costs
 * measured on MI355X (csrc/microbench/unit_costs.hip): per C tile and K-step,
 * in shader-clock cycles,
 *   mfma   = n_mfma * 32 / 4                    matrix pipes (32 cycles per unit of 32768 flop, 4 SIMDs)
 *   valu   = (n_mfma * 17 + n_decode * 6.5 + n_addr * 4) / 4
 *                                               VALU issue ports: an MFMA blocks its SIMD's port for
 *                                               17 of its 32 cycles; a decode instruction costs 6.5
 *   lds    = 4.7 n_b128_reads + 4.6 n_tr_reads + bytes_written / 76
 *   vmem   = bytes_requested / 64
 *   steady = max of the four / 0.85             (II; 0.85 = co-issue efficiency, one global constant)
 *   switch = (120 + 4.7 * first-band reads + 150) / waves per SIMD
 *                                               prolog (LDS latency, Eq. 4 form) + epilog (barrier)
 *   kstep  = steady + rho * switch              (Eq. 9; workgroups sharing a CU overlap, Eq. 10)
 * (n_mfma counts units of 32 x 32 x 16 = 32768 flop: one v_mfma_f32_32x32x16_bf16 or two
 * v_mfma_f32_16x16x32_bf16, which cost the same pipe and port cycles.)
 * mfma_util = mfma / kstep; the chip is power-limited under this kernel, the
 * measured clock follows c * mfma_util^-0.617 (capped at 2.4 GHz) with c = 1.339 GHz for
 * instances that multiply with the 32 x 32 x 16 form and 1.45 GHz for the 16 x 16 x 32
 * form, which draws less power per flop, and
 * pred_flops = flop per K-step * CUs / (kstep / clock).
 * Predicts the full-load throughput of the compiled instances within 15 %
 * from the tile factors and the wave grid alone (measured values: tests/measured/mi355x_instances.txt);
 * it does not see pipeline stalls of a particular schedule. */
typedef struct atb_micro_model {
    double n_mfma;         /* MFMA units (32768 flop) per C tile and K-step */
    double mfma_cycles, valu_cycles, lds_cycles, vmem_cycles;
    double steady_cycles;  /* II of one K-step */
    double switch_cycles;  /* prolog + epilog of one microkernel call */
    double kstep_cycles;
    double mfma_util;      /* predicted share of cycles the matrix pipes are busy */
    double clock_hz;       /* predicted shader clock under that load */
    double pred_flops;     /* whole chip, full load */
} atb_micro_model;

/* wave_m x wave_n: the wave grid of the workgroup (64-lane waves); wg_per_cu:
 * workgroups that share a CU; mfma_rows: 16 or 32, the form of the MFMA.
 * ATB_ERR_INVALID_ARG / ATB_ERR_BAD_TILE if the factors do not divide (32-row
 * bands per wave row, 32-column bands per wave column, T_K % 16). */
atb_status atb_model_microkernel(int T_MA, int T_MC, int T_K, int T_N, int wave_m, int wave_n,
                                 int wg_per_cu, int mfma_rows, atb_micro_model *out);

/* Wave grid, residency and MFMA form of compiled instance `index` (inputs of the call above;
 * any of the four pointers may be NULL). */
atb_status atb_instance_geometry(int index, int *wave_m, int *wave_n, int *wg_per_cu, int *mfma_rows);

/* ------------------------------------------------------- measurement aid */

/* An MFMA-only loop on register operands (no memory traffic, no LDS), for
 * benches that quote the GEMM against what the matrix pipes of this chip
 * sustain in practice as well as against the nominal peak (the nominal figure
 * assumes a clock the chip does not hold under full matrix load).  Not a step
 * of the GEMM.
 * Launches `workgroups` workgroups of 8 waves (two per SIMD, as the GEMM's
 * large tiles); each wave issues iters * 32 v_mfma_f32_32x32x16_bf16
 * (mfma_rows = 32) or iters * 64 v_mfma_f32_16x16x32_bf16 (mfma_rows = 16:
 * the same flop; the form the large GEMM tiles use, and the one that draws
 * less power) on
 * operands that rotate over four register sets; random_operands != 0 fills
 * them with pseudo-random bf16 (random sign and mantissa, exponents 2^-7 .. 2),
 * 0 with the constant 1.0 (which draws less power, hence a higher clock).
 * sink_dev: DEVICE, at least workgroups * 512 * 4 bytes, overwritten (keeps the
 * arithmetic alive).  clocks_dev: DEVICE or NULL; two uint64 written by the
 * first wave: the kernel's length in ticks of the shader-clock counter
 * (s_memtime; measured on MI355X: one tick per two shader cycles) and of the
 * constant-rate counter (s_memrealtime).
 * *flop (HOST, may be NULL) receives the floating-point operations of the
 * launch.  Async on hip_stream; workgroups in [1, 65536], iters in [1, 2^20],
 * mfma_rows 16 or 32 (anything else: ATB_ERR_INVALID_ARG). */
atb_status atb_mfma_probe(void *sink_dev, void *clocks_dev, int workgroups, int iters,
                          int random_operands, int mfma_rows, void *hip_stream, double *flop);

#ifdef __cplusplus
}
#endif
#endif /* ATB_H */
