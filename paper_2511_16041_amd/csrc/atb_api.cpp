// C ABI of libatb (see include/atb.h): argument checking, plans, launches.
#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <new>

#include "atb_internal.h"

struct atb_gemm {
    int64_t M, N, K;
    int instance;
    int b_format, c_format;
    atb_bfp16_layout_t layout;     // A
    atb_bfp16_layout_t layout_b;   // B^T when b_format is BFP16
    atb_bfp16_layout_t layout_c;   // C when c_format is BFP16
    atb::GemmParams proto;   // everything but the pointers
};

namespace {

thread_local int g_last_hip_error = 0;

atb_status hip_status(hipError_t e)
{
    if (e == hipSuccess) return ATB_OK;
    g_last_hip_error = (int)e;
    return ATB_ERR_HIP;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

extern "C" const char *atb_status_string(atb_status s)
{
    switch (s) {
        case ATB_OK: return "ok";
        case ATB_ERR_INVALID_ARG: return "invalid argument";
        case ATB_ERR_BAD_TILE: return "tile factors are not a compiled instance (or T_MC % T_MA != 0)";
        case ATB_ERR_LDS_BUDGET: return "tile buffers exceed the LDS of a compute unit";
        case ATB_ERR_REG_BUDGET: return "C tile exceeds the accumulator registers";
        case ATB_ERR_HIP: return "HIP call failed";
        case ATB_ERR_NOMEM: return "out of host memory";
    }
    return "unknown status";
}

extern "C" int atb_last_hip_error(void) { return g_last_hip_error; }

extern "C" int atb_instance_count(void) { return atb::instance_count(); }

extern "C" atb_status atb_instance_get(int index, int *T_MA, int *T_MC, int *T_K, int *T_N)
{
    if (index < 0 || index >= atb::instance_count()) return ATB_ERR_INVALID_ARG;
    const atb::Instance &x = atb::instance(index);
    if (T_MA) *T_MA = x.T_MA;
    if (T_MC) *T_MC = x.T_MC;
    if (T_K) *T_K = x.T_K;
    if (T_N) *T_N = x.T_N;
    return ATB_OK;
}

extern "C" atb_status atb_bfp16_layout(int64_t M, int64_t K, atb_bfp16_layout_t *out)
{
    if (!out || M < 1 || K < 8 || (K % 8) != 0) return ATB_ERR_INVALID_ARG;
    out->panel_k = atb::kPanelK;
    out->panels = (K + atb::kPanelK - 1) / atb::kPanelK;
    out->man_stride = M * atb::kPanelK;
    out->exp_stride = M * (atb::kPanelK / 8);
    out->exp_off = atb::round_up(out->panels * out->man_stride, 256);
    out->bytes = atb::round_up(out->exp_off + out->panels * out->exp_stride, 256);
    return ATB_OK;
}

extern "C" size_t atb_bfp16_bytes(int64_t M, int64_t K)
{
    atb_bfp16_layout_t l;
    if (atb_bfp16_layout(M, K, &l) != ATB_OK) return 0;
    return (size_t)l.bytes;
}

extern "C" atb_status atb_bfp16_quantize(const float *A, int64_t lda, void *A_bfp, int64_t M, int64_t K,
                                         void *stream)
{
    atb_bfp16_layout_t l;
    if (!A || !A_bfp || atb_bfp16_layout(M, K, &l) != ATB_OK || lda < K || (lda % 4) != 0) return ATB_ERR_INVALID_ARG;
    if (!aligned16(A) || !aligned16(A_bfp)) return ATB_ERR_INVALID_ARG;
    if (M * l.panels * 4 > (int64_t)0x7FFFFFFF * 256) return ATB_ERR_INVALID_ARG;
    int8_t *Am = static_cast<int8_t *>(A_bfp);
    uint8_t *Ae = static_cast<uint8_t *>(A_bfp) + l.exp_off;
    return hip_status(atb::launch_quantize(A, lda, Am, Ae, M, K, static_cast<hipStream_t>(stream)));
}

extern "C" atb_status atb_bfp16_decode(const void *A_bfp, void *A_bf16, int64_t M, int64_t K, void *stream)
{
    atb_bfp16_layout_t l;
    if (!A_bfp || !A_bf16 || atb_bfp16_layout(M, K, &l) != ATB_OK) return ATB_ERR_INVALID_ARG;
    if (!aligned16(A_bfp) || !aligned16(A_bf16)) return ATB_ERR_INVALID_ARG;
    const int8_t *Am = static_cast<const int8_t *>(A_bfp);
    const uint8_t *Ae = static_cast<const uint8_t *>(A_bfp) + l.exp_off;
    return hip_status(atb::launch_decode(Am, Ae, static_cast<uint16_t *>(A_bf16), M, K, static_cast<hipStream_t>(stream)));
}

extern "C" atb_status atb_gemm_create(atb_gemm **out, int64_t M, int64_t N, int64_t K,
                                      int T_MA, int T_MC, int T_K, int T_N)
{
    return atb_gemm_create_fmt(out, M, N, K, T_MA, T_MC, T_K, T_N, ATB_FMT_BF16, ATB_FMT_BF16);
}

extern "C" atb_status atb_gemm_create_fmt(atb_gemm **out, int64_t M, int64_t N, int64_t K,
                                          int T_MA, int T_MC, int T_K, int T_N,
                                          atb_format b_format, atb_format c_format)
{
    if (!out) return ATB_ERR_INVALID_ARG;
    *out = nullptr;
    if (M < 1 || N < 1 || K < 8 || (K % 8) != 0) return ATB_ERR_INVALID_ARG;
    if ((b_format != ATB_FMT_BF16 && b_format != ATB_FMT_BFP16 && b_format != ATB_FMT_BF16_T) ||
        (c_format != ATB_FMT_BF16 && c_format != ATB_FMT_BFP16))
        return ATB_ERR_INVALID_ARG;
    if (b_format == ATB_FMT_BF16_T && c_format != ATB_FMT_BF16) return ATB_ERR_INVALID_ARG;
    const bool other_fmt = (b_format != ATB_FMT_BF16 || c_format != ATB_FMT_BF16);
    if (c_format == ATB_FMT_BFP16 && (N % 8) != 0) return ATB_ERR_INVALID_ARG;   // whole blocks along N
    if (N * atb::round_up(K, 64) >= ((int64_t)1 << 31) || M * atb::round_up(N, 64) >= ((int64_t)1 << 31))
        return ATB_ERR_INVALID_ARG;
    // 32-bit element offsets inside the kernel: keep every plane below 2^31 elements
    if (M > (1 << 23) || N > (1 << 23) || K > (1 << 24) || M * N >= ((int64_t)1 << 31) ||
        M * atb::round_up(K, 64) >= ((int64_t)1 << 31) || K * N >= ((int64_t)1 << 31))
        return ATB_ERR_INVALID_ARG;
    if (T_MA < 1 || T_MC < 1 || T_K < 1 || T_N < 1) return ATB_ERR_INVALID_ARG;
    if (T_MC % T_MA != 0) return ATB_ERR_BAD_TILE;
    // byte offsets of a B tile's requests relative to its first row are 32-bit
    if (N * ((int64_t)T_K + 1) * 2 >= ((int64_t)1 << 31)) return ATB_ERR_INVALID_ARG;
    // budgets of one CU: A (double-buffered, bf16) and B (double-buffered, bf16) in 160 KiB of LDS,
    // the fp32 C tile in 4 waves x 256 accumulator registers
    if ((int64_t)4 * T_MC * T_N > 256 * 1024) return ATB_ERR_REG_BUDGET;
    if ((int64_t)2 * 2 * T_MA * T_K + (int64_t)2 * 2 * T_K * T_N > 160 * 1024) return ATB_ERR_LDS_BUDGET;
    const int idx = atb::find_instance(T_MA, T_MC, T_K, T_N);
    if (idx < 0) return ATB_ERR_BAD_TILE;
    if (other_fmt && atb::instance(idx).launch_fmt == nullptr) return ATB_ERR_BAD_TILE;
    if (b_format == ATB_FMT_BF16_T) {
        if (!atb::instance(idx).has_b_transposed) return ATB_ERR_BAD_TILE;
        // byte offsets of a B^T tile's requests relative to its first row are 32-bit
        if ((int64_t)2 * T_N * K >= ((int64_t)1 << 31)) return ATB_ERR_INVALID_ARG;
    }

    atb_gemm *g = new (std::nothrow) atb_gemm;
    if (!g) return ATB_ERR_NOMEM;
    g->M = M; g->N = N; g->K = K;
    g->instance = idx;
    g->b_format = (int)b_format;
    g->c_format = (int)c_format;
    atb_bfp16_layout(M, K, &g->layout);
    atb_bfp16_layout(N, K, &g->layout_b);
    g->layout_c = atb_bfp16_layout_t{0, 0, 0, 0, 0, 0};
    if (c_format == ATB_FMT_BFP16) atb_bfp16_layout(M, N, &g->layout_c);
    atb::GemmParams &p = g->proto;
    p.Am = nullptr; p.Ae = nullptr; p.B = nullptr; p.C = nullptr;
    p.Bm = nullptr; p.Be = nullptr; p.Cm = nullptr; p.Ce = nullptr;
    p.k_panels = (int)g->layout.panels;
    p.n_panels = (int)g->layout_c.panels;
    p.M = (int)M; p.N = (int)N; p.K = (int)K;
    p.tiles_m = (int)((M + T_MC - 1) / T_MC);
    p.tiles_n = (int)((N + T_N - 1) / T_N);
    // C in BFP16: the tiles also cover the zero tail of C's last panel (columns N .. 64 * panels - 1),
    // so that the result can be the BFP16 operand of a following GEMM as it is
    if (c_format == ATB_FMT_BFP16) p.tiles_n = (int)((atb::round_up(N, atb::kPanelK) + T_N - 1) / T_N);
    p.group_m = (int)std::max<int64_t>(1, 2048 / T_MC);   // an XCD's patch of C tiles is 2048 rows high
    // measurement aid: ATB_GROUP_M=<tile rows> overrides the height of the patch, so that the counters can
    // be read with the tiles resident on an XCD laid out as one row (1) or one column (>= 32) of C tiles
    if (const char *gm = std::getenv("ATB_GROUP_M"); gm && gm[0]) {
        const long v = std::strtol(gm, nullptr, 10);
        if (v >= 1 && v <= 65536) p.group_m = (int)v;   // anything else is ignored
    }
    if (const char *log = std::getenv("ATB_LOG"); log && log[0] == '1') {
        const atb::Instance &x = atb::instance(idx);
        std::fprintf(stderr, "atb_gemm_create: M=%lld N=%lld K=%lld T_MA=%d T_MC=%d T_K=%d T_N=%d rho=%d b=%s c=%s "
                             "instance=%d waves=%dx%d threads=%d lds=%d tiles=%dx%d group_m=%d k_panels=%d\n",
                     (long long)M, (long long)N, (long long)K, T_MA, T_MC, T_K, T_N, T_MC / T_MA,
                     b_format == ATB_FMT_BFP16 ? "bfp16" : b_format == ATB_FMT_BF16_T ? "bf16_t" : "bf16", c_format == ATB_FMT_BFP16 ? "bfp16" : "bf16", idx,
                     x.wave_m, x.wave_n, x.threads, x.lds_bytes, p.tiles_m, p.tiles_n, p.group_m, p.k_panels);
    }
    *out = g;
    return ATB_OK;
}

extern "C" atb_status atb_gemm_run(const atb_gemm *g, const void *A_bfp, const void *B, void *C, void *stream)
{
    if (!g || !A_bfp || !B || !C) return ATB_ERR_INVALID_ARG;
    if (!aligned16(A_bfp) || !aligned16(B) || !aligned16(C)) return ATB_ERR_INVALID_ARG;
    atb::GemmParams p = g->proto;
    p.Am = static_cast<const int8_t *>(A_bfp);
    p.Ae = static_cast<const uint8_t *>(A_bfp) + g->layout.exp_off;
    if (g->b_format == ATB_FMT_BFP16) {
        p.Bm = static_cast<const int8_t *>(B);
        p.Be = static_cast<const uint8_t *>(B) + g->layout_b.exp_off;
    } else {
        p.B = static_cast<const uint16_t *>(B);
    }
    if (g->c_format == ATB_FMT_BFP16) {
        p.Cm = static_cast<int8_t *>(C);
        p.Ce = static_cast<uint8_t *>(C) + g->layout_c.exp_off;
    } else {
        p.C = static_cast<uint16_t *>(C);
    }
    const atb::Instance &x = atb::instance(g->instance);
    if (g->b_format != ATB_FMT_BF16 || g->c_format != ATB_FMT_BF16)
        return hip_status(x.launch_fmt(p, g->b_format, g->c_format, static_cast<hipStream_t>(stream)));
    return hip_status(x.launch(p, static_cast<hipStream_t>(stream)));
}

extern "C" void atb_gemm_destroy(atb_gemm *g) { delete g; }

extern "C" atb_status atb_gemm_launch_info(const atb_gemm *g, int64_t *workgroups, int *threads, int *lds_bytes)
{
    if (!g) return ATB_ERR_INVALID_ARG;
    const atb::Instance &x = atb::instance(g->instance);
    const int64_t total = (int64_t)g->proto.tiles_m * g->proto.tiles_n;
    if (workgroups) *workgroups = (total + 7) / 8 * 8;
    if (threads) *threads = x.threads;
    if (lds_bytes) *lds_bytes = x.lds_bytes;
    return ATB_OK;
}

extern "C" atb_status atb_mfma_probe(void *sink, void *clocks, int workgroups, int iters, int random_operands,
                                     int mfma_rows, void *stream, double *flop)
{
    if (!sink || workgroups < 1 || workgroups > 65536 || iters < 1 || iters > (1 << 20)) return ATB_ERR_INVALID_ARG;
    if (mfma_rows != 16 && mfma_rows != 32) return ATB_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(sink) & 3u) != 0 || (reinterpret_cast<uintptr_t>(clocks) & 7u) != 0) return ATB_ERR_INVALID_ARG;
    if (flop) *flop = atb::mfma_probe_flop(workgroups, iters);
    return hip_status(atb::launch_mfma_probe(static_cast<float *>(sink), static_cast<unsigned long long *>(clocks), workgroups,
                                             iters, random_operands != 0, mfma_rows, static_cast<hipStream_t>(stream)));
}
