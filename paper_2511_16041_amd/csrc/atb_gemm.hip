// BFP16 x BF16 GEMM with asymmetric tile buffering for gfx950 (MI355X).
//
// One workgroup owns one T_MC x T_N tile of C for the whole reduction
// (output-stationary schedule, Sec. 3.1 of arXiv 2511.16041) and walks the ATB
// loop nest of Sec. 3 / Sec. 5:
//
//   for kt in K-steps of T_K:                    B tile T_K x T_N resident
//     for s in 0 .. rho-1 (rho = T_MC / T_MA):   A sub-tile T_MA x T_K
//        "microkernel": C[s*T_MA : +T_MA, :] += A_sub * B_tile
//
// Mapping onto a CU:
//   * the C tile lives in MFMA accumulator registers (fp32), spread over a
//     WM x WN grid of 64-lane waves; 32-row bands of the tile are dealt
//     round-robin to the WM wave rows so that every A sub-tile feeds all waves;
//   * each wave keeps its slice of the B tile in VGPRs for the whole K-step
//     (loaded once from LDS), so the rho microkernels of a K-step re-use B
//     from registers -- the register-level form of "B stays resident";
//   * A sub-tiles are fetched from HBM/L2 as raw BFP16 (16 mantissa bytes +
//     2 exponent bytes per lane), decoded to bf16 in registers (exact) and
//     written to a double-buffered LDS area of only T_MA rows;
//   * one workgroup barrier per sub-tile is the "kernel switch" of Sec. 5.
// T_MA == T_MC is the symmetric baseline: same code, one sub-tile per K-step.
//
// MFMA: v_mfma_f32_32x32x16_bf16.  Operand lane layout: lane l supplies row
// (l % 32) of its operand and the 8 consecutive k values 8*(l/32) .. +7, which
// for the A operand is exactly one BFP16 block.  The B fragment is passed as
// the first operand and the A fragment as the second, so a lane of the result
// holds one row m (= l % 32) and 16 columns n = 8*(v/4) + 4*(l/32) + v%4,
// i.e. groups of 4 consecutive columns -> 8-byte bf16 stores.
#include "atb_internal.h"

namespace atb {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef short shortx4 __attribute__((ext_vector_type(4)));

#define ATB_DEV __device__ __forceinline__

// Sign-extended byte `byte` of word w as float (one v_cvt_f32_i32 with a byte select).
ATB_DEV float mant_to_float(int w, int byte) { return (float)(int)(signed char)(w >> (8 * byte)); }

// 8 int8 mantissas (two dwords) with shift s = E - 133  ->  8 bf16, exact:
// |m| <= 127 has at most 7 significant bits, bf16 keeps 8.
ATB_DEV bf16x8 decode_block(int w0, int w1, int shift)
{
    bf16x8 r;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        r[t] = (__bf16)ldexpf(mant_to_float(w0, t), shift);
        r[4 + t] = (__bf16)ldexpf(mant_to_float(w1, t), shift);
    }
    return r;
}

template <int T_MA_, int T_MC_, int T_K_, int T_N_, int WM_, int WN_, int BMODE_>
struct Shape {
    static constexpr int T_MA = T_MA_, T_MC = T_MC_, T_K = T_K_, T_N = T_N_, WM = WM_, WN = WN_;
    static constexpr int BMODE = BMODE_;          // 0: B transposed into LDS; 1: row-major LDS + transposing reads
    static constexpr int NT = WM * WN * 64;       // threads
    static constexpr int RHO = T_MC / T_MA;
    static constexpr int MT = T_MC / 32;          // 32-row bands in the C tile
    static constexpr int SMT = T_MA / 32;         // bands per A sub-tile
    static constexpr int MTW = MT / WM;           // bands per wave
    static constexpr int NTW = T_N / 32 / WN;     // 32-column bands per wave
    static constexpr int KS = T_K / 16;           // MFMA k-slices per K-step
    static constexpr bool BALANCED = (SMT % WM) == 0;
    // LDS pitches in bytes.  +16 bytes per row de-phases the banks for the 16-byte fragment reads.
    static constexpr int PA = T_K * 2 + 16;
    static constexpr int PB = (BMODE == 1) ? (T_N * 2 + 64) : (T_K * 2 + 16);
    static constexpr int A_BYTES = T_MA * PA;
    static constexpr int B_BYTES = (BMODE == 1) ? T_K * PB : T_N * PB;
    static constexpr int LDS_BYTES = 2 * A_BYTES + 2 * B_BYTES;
    // staging work per thread
    static constexpr int A_CHUNKS = T_MA * (T_K / 16);               // 16 mantissas per chunk
    static constexpr int A_PER_THREAD = (A_CHUNKS + NT - 1) / NT;
    static constexpr int B_CHUNKS = T_K * (T_N / 8);                 // 8 bf16 per chunk
    static constexpr int B_PER_THREAD = (B_CHUNKS + NT - 1) / NT;
    static_assert(T_MC % T_MA == 0, "rho must be an integer");
    static_assert(T_MA % 32 == 0 && T_N % (32 * WN) == 0 && T_K % 16 == 0, "MFMA 32x32x16 granularity");
    static_assert(MT % WM == 0, "bands must split evenly over wave rows");
    static_assert(BALANCED || (WM % SMT) == 0, "sub-tile bands must divide the wave rows");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget of a gfx950 CU");
    static_assert(MTW * NTW * 16 <= 256, "C tile must fit the accumulator registers");
};

// Raw A sub-tile held in registers between the global load and the decode.
template <class S>
struct ARegs {
    int4 mant[S::A_PER_THREAD];
    unsigned expo[S::A_PER_THREAD];
};

template <class S>
struct BRegs {
    int4 v[S::B_PER_THREAD];
};

// Global -> registers: raw BFP16 of A rows [row0, row0 + T_MA), k in [k0, k0 + T_K).
template <class S>
ATB_DEV void load_a_global(const GemmParams &p, int row0, int k0, int tid, ARegs<S> &r)
{
#pragma unroll
    for (int i = 0; i < S::A_PER_THREAD; ++i) {
        const int c = tid + i * S::NT;
        const int row = c / (S::T_K / 16), q = c % (S::T_K / 16);
        const int grow = row0 + row, k = k0 + q * 16;
        int4 m = make_int4(0, 0, 0, 0);
        unsigned e = 0;
        // ldm is a multiple of 16, so a chunk lies entirely inside or outside a row;
        // the bytes between K and ldm are zero by the layout's contract.
        if (c < S::A_CHUNKS && grow < p.M && k < p.ldm) {
            m = *reinterpret_cast<const int4 *>(p.Am + (int64_t)grow * p.ldm + k);
            e = *reinterpret_cast<const unsigned short *>(p.Ae + (int64_t)grow * p.lde + (k >> 3));
        }
        r.mant[i] = m;
        r.expo[i] = e;
    }
}

// Registers -> decode -> LDS (bf16, [row][k], pitch PA).
template <class S>
ATB_DEV void store_a_lds(char *a_lds, int tid, const ARegs<S> &r)
{
#pragma unroll
    for (int i = 0; i < S::A_PER_THREAD; ++i) {
        const int c = tid + i * S::NT;
        if (c < S::A_CHUNKS) {
            const int row = c / (S::T_K / 16), q = c % (S::T_K / 16);
            const int s0 = (int)(r.expo[i] & 0xFFu) - 133;
            const int s1 = (int)((r.expo[i] >> 8) & 0xFFu) - 133;
            bf16x8 lo = decode_block(r.mant[i].x, r.mant[i].y, s0);
            bf16x8 hi = decode_block(r.mant[i].z, r.mant[i].w, s1);
            char *dst = a_lds + row * S::PA + q * 32;
            *reinterpret_cast<bf16x8 *>(dst) = lo;
            *reinterpret_cast<bf16x8 *>(dst + 16) = hi;
        }
    }
}

// Global -> registers: B rows [k0, k0 + T_K), columns [n0, n0 + T_N), 8 columns per chunk.
template <class S>
ATB_DEV void load_b_global(const GemmParams &p, int k0, int n0, int tid, bool vec_ok, BRegs<S> &r)
{
#pragma unroll
    for (int i = 0; i < S::B_PER_THREAD; ++i) {
        const int c = tid + i * S::NT;
        const int krow = c / (S::T_N / 8), nc = c % (S::T_N / 8);
        const int k = k0 + krow, n = n0 + nc * 8;
        int4 v = make_int4(0, 0, 0, 0);
        if (c < S::B_CHUNKS && k < p.K && n < p.N) {
            const uint16_t *src = p.B + (int64_t)k * p.N + n;
            if (vec_ok && n + 8 <= p.N) {
                v = *reinterpret_cast<const int4 *>(src);
            } else {
                // ragged right edge or a row pitch that is not 16-byte aligned
                unsigned short t[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) t[j] = (n + j < p.N) ? src[j] : (unsigned short)0;
                v.x = t[0] | (t[1] << 16);
                v.y = t[2] | (t[3] << 16);
                v.z = t[4] | (t[5] << 16);
                v.w = t[6] | (t[7] << 16);
            }
        }
        r.v[i] = v;
    }
}

template <class S>
ATB_DEV void store_b_lds(char *b_lds, int tid, const BRegs<S> &r)
{
#pragma unroll
    for (int i = 0; i < S::B_PER_THREAD; ++i) {
        const int c = tid + i * S::NT;
        if (c < S::B_CHUNKS) {
            const int krow = c / (S::T_N / 8), nc = c % (S::T_N / 8);
            if constexpr (S::BMODE == 1) {
                *reinterpret_cast<int4 *>(b_lds + krow * S::PB + nc * 16) = r.v[i];
            } else {
                // transposed: [n][k], pitch PB
                const int w[4] = {r.v[i].x, r.v[i].y, r.v[i].z, r.v[i].w};
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    unsigned short h = (unsigned short)((unsigned)w[j >> 1] >> (16 * (j & 1)));
                    *reinterpret_cast<unsigned short *>(b_lds + (nc * 8 + j) * S::PB + krow * 2) = h;
                }
            }
        }
    }
}

// LDS -> the wave's B fragments for one K-step: frag[ks][nt] holds, per lane l,
// column (wn*NTW + nt)*32 + l%32 and k = ks*16 + 8*(l/32) .. +7.
template <class S>
ATB_DEV void read_b_frags(const char *b_lds, int wn, int lane, bf16x8 (&frag)[S::KS][S::NTW])
{
#pragma unroll
    for (int ks = 0; ks < S::KS; ++ks) {
#pragma unroll
        for (int nt = 0; nt < S::NTW; ++nt) {
            const int nbase = (wn * S::NTW + nt) * 32;
            if constexpr (S::BMODE == 1) {
                // Transposing read: within each group of 16 lanes, lane i addresses 4 consecutive
                // columns of row i/4; lane j receives column j of those 4 rows.
                const int blk = lane >> 4, j = lane & 15;
                const int krow = ks * 16 + 8 * (blk >> 1) + (j >> 2);
                const int ncol = nbase + 16 * (blk & 1) + 4 * (j & 3);
                const char *src = b_lds + krow * S::PB + ncol * 2;
                typedef __attribute__((address_space(3))) shortx4 lds_shortx4;
                shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_shortx4 *)(src));
                shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_shortx4 *)(src + 4 * S::PB));
                union { shortx4 s[2]; bf16x8 b; } u;
                u.s[0] = lo;
                u.s[1] = hi;
                frag[ks][nt] = u.b;
            } else {
                const int n = nbase + (lane & 31);
                frag[ks][nt] = *reinterpret_cast<const bf16x8 *>(b_lds + n * S::PB + ks * 32 + (lane >> 5) * 16);
            }
        }
    }
}

// One microkernel: the bands of sub-tile `s` that belong to this wave row.
template <class S, int s>
ATB_DEV void microkernel(const char *a_lds, int wm, int lane, const bf16x8 (&bfrag)[S::KS][S::NTW],
                         floatx16 (&acc)[S::MTW][S::NTW])
{
    if constexpr (S::BALANCED) {
        constexpr int PER = S::SMT / S::WM;       // bands of this sub-tile per wave row
#pragma unroll
        for (int il = 0; il < PER; ++il) {
            const int band = il * S::WM + wm;     // band inside the sub-tile
            constexpr int dummy = 0;
            (void)dummy;
            const int local = (s * S::SMT) / S::WM + il;   // accumulator band of this wave (compile time)
            const char *src = a_lds + (band * 32 + (lane & 31)) * S::PA + (lane >> 5) * 16;
            bf16x8 afrag[S::KS];
#pragma unroll
            for (int ks = 0; ks < S::KS; ++ks) afrag[ks] = *reinterpret_cast<const bf16x8 *>(src + ks * 32);
#pragma unroll
            for (int ks = 0; ks < S::KS; ++ks)
#pragma unroll
                for (int nt = 0; nt < S::NTW; ++nt)
                    acc[local][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfrag[ks][nt], afrag[ks],
                                                                            acc[local][nt], 0, 0, 0);
        }
    } else {
        // fewer bands in a sub-tile than wave rows: band i of sub-tile s belongs to wave row (s*SMT+i) % WM
#pragma unroll
        for (int i = 0; i < S::SMT; ++i) {
            constexpr int dummy = 0;
            (void)dummy;
            const int mt = s * S::SMT + i;        // compile time
            if ((mt % S::WM) == wm) {
                const int local = mt / S::WM;
                const char *src = a_lds + (i * 32 + (lane & 31)) * S::PA + (lane >> 5) * 16;
                bf16x8 afrag[S::KS];
#pragma unroll
                for (int ks = 0; ks < S::KS; ++ks) afrag[ks] = *reinterpret_cast<const bf16x8 *>(src + ks * 32);
#pragma unroll
                for (int ks = 0; ks < S::KS; ++ks)
#pragma unroll
                    for (int nt = 0; nt < S::NTW; ++nt)
                        acc[local][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfrag[ks][nt], afrag[ks],
                                                                                acc[local][nt], 0, 0, 0);
            }
        }
    }
}

// Row inside the C tile of accumulator band `local` of wave row wm.
// Bands are dealt round-robin: band mt belongs to wave row mt % WM.
template <class S>
ATB_DEV int band_row(int local, int wm) { return (local * S::WM + wm) * 32; }

template <class S, int s>
ATB_DEV void phases(const GemmParams &p, char *a_lds0, char *a_lds1, char *b_next_lds, int &abuf, int m0,
                    int n0, int k0, int tid, int wm, int lane, bool vec_ok,
                    const bf16x8 (&bfrag)[S::KS][S::NTW], floatx16 (&acc)[S::MTW][S::NTW], BRegs<S> &breg)
{
    if constexpr (s < S::RHO) {
        // prefetch the next A sub-tile: (kt, s+1), or (kt+1, 0) after the last one
        ARegs<S> areg;
        constexpr bool last = (s + 1 == S::RHO);
        const int next_row0 = m0 + (last ? 0 : (s + 1) * S::T_MA);
        const int next_k0 = last ? k0 + S::T_K : k0;
        load_a_global<S>(p, next_row0, next_k0, tid, areg);
        if constexpr (s == 0) load_b_global<S>(p, k0 + S::T_K, n0, tid, vec_ok, breg);

        char *a_cur = abuf ? a_lds1 : a_lds0;
        char *a_nxt = abuf ? a_lds0 : a_lds1;
        microkernel<S, s>(a_cur, wm, lane, bfrag, acc);

        store_a_lds<S>(a_nxt, tid, areg);
        if constexpr (last) store_b_lds<S>(b_next_lds, tid, breg);
        __syncthreads();                          // the "kernel switch" of the ATB nest
        abuf ^= 1;
        phases<S, s + 1>(p, a_lds0, a_lds1, b_next_lds, abuf, m0, n0, k0, tid, wm, lane, vec_ok, bfrag, acc, breg);
    }
}

template <class S>
__global__ void __launch_bounds__(S::NT) atb_gemm_kernel(const GemmParams p)
{
    __shared__ __attribute__((aligned(16))) char lds[S::LDS_BYTES];
    char *a_lds0 = lds, *a_lds1 = lds + S::A_BYTES;
    char *b_lds0 = lds + 2 * S::A_BYTES, *b_lds1 = b_lds0 + S::B_BYTES;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave % S::WM, wn = wave / S::WM;

    // Workgroup -> C tile.  Workgroups are dealt round-robin to the 8 XCDs (each with its own L2);
    // give each XCD a contiguous run of tiles, and walk tiles in bands of group_m tile rows so that
    // the workgroups resident on one XCD share few distinct A row panels and B column panels.
    const int total = p.tiles_m * p.tiles_n;
    const int per_xcd = (total + 7) / 8;
    const int logical = (int)(blockIdx.x % 8) * per_xcd + (int)(blockIdx.x / 8);
    if (logical >= total) return;
    const int band_sz = p.group_m * p.tiles_n;
    const int band = logical / band_sz, in_band = logical % band_sz;
    const int rows_here = min(p.group_m, p.tiles_m - band * p.group_m);
    const int tm = band * p.group_m + in_band % rows_here;
    const int tn = in_band / rows_here;
    const int m0 = tm * S::T_MC, n0 = tn * S::T_N;

    const bool vec_ok = (p.N % 8) == 0;
    const int KT = (p.K + S::T_K - 1) / S::T_K;

    floatx16 acc[S::MTW][S::NTW];
#pragma unroll
    for (int a = 0; a < S::MTW; ++a)
#pragma unroll
        for (int b = 0; b < S::NTW; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.0f;

    // prologue: first B tile and first A sub-tile
    {
        BRegs<S> b0;
        ARegs<S> a0;
        load_b_global<S>(p, 0, n0, tid, vec_ok, b0);
        load_a_global<S>(p, m0, 0, tid, a0);
        store_b_lds<S>(b_lds0, tid, b0);
        store_a_lds<S>(a_lds0, tid, a0);
    }
    __syncthreads();

    int abuf = 0;
    for (int kt = 0; kt < KT; ++kt) {
        const char *b_cur = (kt & 1) ? b_lds1 : b_lds0;
        char *b_nxt = (kt & 1) ? b_lds0 : b_lds1;
        bf16x8 bfrag[S::KS][S::NTW];
        read_b_frags<S>(b_cur, wn, lane, bfrag);
        BRegs<S> breg;
        phases<S, 0>(p, a_lds0, a_lds1, b_nxt, abuf, m0, n0, kt * S::T_K, tid, wm, lane, vec_ok, bfrag, acc, breg);
    }

    // epilogue: fp32 -> bf16 (round to nearest even) and store, once per tile
    const bool st_vec = (p.N % 4) == 0;
#pragma unroll
    for (int a = 0; a < S::MTW; ++a) {
        const int m = m0 + band_row<S>(a, wm) + (lane & 31);
#pragma unroll
        for (int b = 0; b < S::NTW; ++b) {
            const int nb = n0 + (wn * S::NTW + b) * 32 + 4 * (lane >> 5);
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int n = nb + 8 * g;
                bf16x4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = (__bf16)acc[a][b][4 * g + e];
                if (m < p.M && n < p.N) {
                    uint16_t *dst = p.C + (int64_t)m * p.N + n;
                    if (st_vec && n + 4 <= p.N) {
                        *reinterpret_cast<bf16x4 *>(dst) = o;
                    } else {
                        union { bf16x4 v; uint16_t h[4]; } u;
                        u.v = o;
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (n + e < p.N) dst[e] = u.h[e];
                    }
                }
            }
        }
    }
}

template <class S>
hipError_t launch_instance(const GemmParams &p, hipStream_t stream)
{
    const int total = p.tiles_m * p.tiles_n;
    const int per_xcd = (total + 7) / 8;
    hipLaunchKernelGGL((atb_gemm_kernel<S>), dim3(per_xcd * 8), dim3(S::NT), 0, stream, p);
    return hipGetLastError();
}

template <class S>
Instance make_instance()
{
    Instance i;
    i.T_MA = S::T_MA;
    i.T_MC = S::T_MC;
    i.T_K = S::T_K;
    i.T_N = S::T_N;
    i.wave_m = S::WM;
    i.wave_n = S::WN;
    i.threads = S::NT;
    i.lds_bytes = S::LDS_BYTES;
    i.launch = &launch_instance<S>;
    return i;
}

#ifndef ATB_BMODE
#define ATB_BMODE 0
#endif

const Instance g_instances[] = {
    // T_MC = T_N = 256, T_K = 64: the sweep over rho = 1, 2, 4, 8
    make_instance<Shape<256, 256, 64, 256, 2, 2, ATB_BMODE>>(),
    make_instance<Shape<128, 256, 64, 256, 2, 2, ATB_BMODE>>(),
    make_instance<Shape<64, 256, 64, 256, 2, 2, ATB_BMODE>>(),
    make_instance<Shape<32, 256, 64, 256, 1, 4, ATB_BMODE>>(),
    // small tiles for small problems
    make_instance<Shape<64, 64, 64, 64, 2, 2, ATB_BMODE>>(),
    make_instance<Shape<32, 64, 64, 64, 2, 2, ATB_BMODE>>(),
};

}  // namespace

int instance_count() { return (int)(sizeof(g_instances) / sizeof(g_instances[0])); }
const Instance &instance(int i) { return g_instances[i]; }
int find_instance(int T_MA, int T_MC, int T_K, int T_N)
{
    for (int i = 0; i < instance_count(); ++i) {
        const Instance &x = g_instances[i];
        if (x.T_MA == T_MA && x.T_MC == T_MC && x.T_K == T_K && x.T_N == T_N) return i;
    }
    return -1;
}

}  // namespace atb
