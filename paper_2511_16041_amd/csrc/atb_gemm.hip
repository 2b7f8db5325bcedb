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

template <int T_MA_, int T_MC_, int T_K_, int T_N_, int WM_, int WN_, int PF_>
struct Shape {
    static constexpr int T_MA = T_MA_, T_MC = T_MC_, T_K = T_K_, T_N = T_N_, WM = WM_, WN = WN_;
    static constexpr int PF = PF_;                // A sub-tiles fetched this many phases ahead of their use
    static constexpr int NT = WM * WN * 64;       // threads
    static constexpr int RHO = T_MC / T_MA;
    static constexpr int MT = T_MC / 32;          // 32-row bands in the C tile
    static constexpr int SMT = T_MA / 32;         // bands per A sub-tile
    static constexpr int MTW = MT / WM;           // bands per wave
    static constexpr int NTW = T_N / 32 / WN;     // 32-column bands per wave
    static constexpr int KS = T_K / 16;           // MFMA k-slices per K-step
    static constexpr int PER = SMT / WM;          // bands of one sub-tile per wave row
    static constexpr int NM = PER * KS * NTW;     // MFMAs per wave per microkernel
    // LDS pitches in bytes.  The pad de-phases the banks for the fragment reads.
    static constexpr int PA = T_K * 2 + 16;
    static constexpr int PB = T_N * 2 + 64;
    static constexpr int A_BYTES = T_MA * PA;
    static constexpr int B_BYTES = T_K * PB;
    static constexpr int LDS_BYTES = 2 * A_BYTES + 2 * B_BYTES;
    // staging work per thread: A in chunks of ACE mantissas (ACE/8 BFP16 blocks), B in chunks of 8 bf16
    static constexpr int ACE = (T_MA * T_K / NT >= 16) ? 16 : 8;
    static constexpr int A_CHUNKS = T_MA * T_K / ACE;
    static constexpr int A_PER_THREAD = A_CHUNKS / NT;
    static constexpr int A_CPR = T_K / ACE;       // chunks per A row
    static constexpr int NPAIR = A_PER_THREAD * ACE / 2;   // pairs of mantissas each thread decodes per sub-tile
    static constexpr int B_CHUNKS = T_K * (T_N / 8);
    static constexpr int B_PER_THREAD = B_CHUNKS / NT;
    static constexpr int B_CPR = T_N / 8;         // chunks per B row
    static_assert(T_MC % T_MA == 0, "rho must be an integer");
    static_assert(PF >= 1 && PF <= 4, "prefetch distance");
    static_assert(T_MA % 32 == 0 && T_N % (32 * WN) == 0 && T_K % 16 == 0, "MFMA 32x32x16 granularity");
    static_assert(MT % WM == 0 && SMT % WM == 0, "every sub-tile must feed every wave row equally");
    static_assert(A_CHUNKS % NT == 0 && NT % A_CPR == 0, "A staging must split evenly over the threads");
    static_assert(B_CHUNKS % NT == 0 && NT % B_CPR == 0, "B staging must split evenly over the threads");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget of a gfx950 CU");
    static_assert(MTW * NTW * 16 <= 256, "C tile must fit the accumulator registers");
};

typedef int intx4 __attribute__((ext_vector_type(4)));
typedef int intx2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// Buffer descriptors (V#) of the three inputs.  A load whose byte offset lies outside
// [0, num_records) returns zero without touching memory, which is what masks the edges.
struct Rsrc {
    __amdgpu_buffer_rsrc_t am, ae, b;
};

constexpr int kRsrcFlags = 0x00020000;           // raw buffer, 32-bit data format
constexpr int kOutOfRange = (int)0x80000000;     // a byte offset no buffer of ours reaches

#define ATB_FENCE() __builtin_amdgcn_sched_barrier(0)

// The per-workgroup state of one C tile.  Everything is indexed with compile-time constants after
// inlining, so the arrays live in registers (acc in AccVGPRs).
template <class S, bool VEC>
struct TileKernel {
    const GemmParams &p;
    Rsrc rs;
    char *a_lds[2];
    char *b_lds[2];
    int tid, lane, wm, wn, m0, n0;
    // per-thread staging coordinates (chunk i adds a compile-time multiple of rows)
    int a_row, a_q, b_row, b_c;

    floatx16 acc[S::MTW][S::NTW];
    bf16x8 bfrag[S::KS][S::NTW];       // this wave's slice of the resident B tile
    bf16x8 afrag[2][S::KS];            // A fragments of the current and the next band
    intx4 a_mant[S::PF][S::A_PER_THREAD];
    unsigned a_expo[S::PF][S::A_PER_THREAD];
    intx4 b_raw[S::B_PER_THREAD];
    unsigned dec[4];                   // bf16 pairs of the BFP16 block being decoded
    int shift;

    ATB_DEV TileKernel(const GemmParams &p_, char *lds, int m0_, int n0_) : p(p_), m0(m0_), n0(n0_)
    {
        a_lds[0] = lds;
        a_lds[1] = lds + S::A_BYTES;
        b_lds[0] = lds + 2 * S::A_BYTES;
        b_lds[1] = b_lds[0] + S::B_BYTES;
        tid = threadIdx.x;
        lane = tid & 63;
        const int wave = tid >> 6;
        wm = wave % S::WM;
        wn = wave / S::WM;
        a_row = tid / S::A_CPR;
        a_q = tid % S::A_CPR;
        b_row = tid / S::B_CPR;
        b_c = tid % S::B_CPR;
        rs.am = __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(p.Am), 0, p.M * p.ldm, kRsrcFlags);
        rs.ae = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(p.Ae), 0, p.M * p.lde, kRsrcFlags);
        rs.b = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(p.B), 0, p.K * p.N * 2, kRsrcFlags);
#pragma unroll
        for (int a = 0; a < S::MTW; ++a)
#pragma unroll
            for (int b = 0; b < S::NTW; ++b)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.0f;
    }

    // ---- global -> registers -------------------------------------------------------------
    // Raw BFP16 of A rows [row0, row0 + T_MA), k in [k0, k0 + T_K) into register set `set`.
    // Rows >= M fall off the end of the planes (zero mantissas); chunks with k >= ldm are sent out
    // of range explicitly; mantissa bytes between K and ldm are zero by the layout's contract.
    template <int set = S::PF - 1>
    ATB_DEV void load_a(int row0, int k0)
    {
#pragma unroll
        for (int i = 0; i < S::A_PER_THREAD; ++i) {
            const int grow = row0 + a_row + i * (S::NT / S::A_CPR);
            const int k = k0 + a_q * S::ACE;
            const bool in = k < p.ldm;
            const int moff = in ? grow * p.ldm + k : kOutOfRange;
            const int eoff = in ? grow * p.lde + (k >> 3) : kOutOfRange;
            if constexpr (S::ACE == 16) {
                a_mant[set][i] = __builtin_amdgcn_raw_buffer_load_b128(rs.am, moff, 0, 0);
                a_expo[set][i] = __builtin_amdgcn_raw_buffer_load_b16(rs.ae, eoff, 0, 0);
            } else {
                intx2 t = __builtin_amdgcn_raw_buffer_load_b64(rs.am, moff, 0, 0);
                a_mant[set][i] = intx4{t.x, t.y, 0, 0};
                a_expo[set][i] = __builtin_amdgcn_raw_buffer_load_b8(rs.ae, eoff, 0, 0);
            }
        }
    }

    // B rows [k0, k0 + T_K), columns [n0, n0 + T_N), 8 columns per chunk.
    // VEC (N % 8 == 0): one 16-byte load per chunk; rows >= K fall off the end of B (zero); columns
    // >= N wrap into the next row, which only feeds output columns that are never stored.
    // !VEC: element loads, each masked.
    ATB_DEV void load_b(int k0)
    {
#pragma unroll
        for (int i = 0; i < S::B_PER_THREAD; ++i) {
            const int k = k0 + b_row + i * (S::NT / S::B_CPR);
            const int n = n0 + b_c * 8;
            if constexpr (VEC) {
                b_raw[i] = __builtin_amdgcn_raw_buffer_load_b128(rs.b, (k * p.N + n) * 2, 0, 0);
            } else {
                unsigned t[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int off = (n + j < p.N) ? (k * p.N + n + j) * 2 : kOutOfRange;
                    t[j] = __builtin_amdgcn_raw_buffer_load_b16(rs.b, off, 0, 0);
                }
                b_raw[i] = intx4{(int)(t[0] | (t[1] << 16)), (int)(t[2] | (t[3] << 16)),
                                 (int)(t[4] | (t[5] << 16)), (int)(t[6] | (t[7] << 16))};
            }
        }
    }

    // ---- registers -> LDS ----------------------------------------------------------------
    // Decode mantissa pair t of chunk i of register set `set` (exact: |m| <= 127 has 7 significant
    // bits, bf16 keeps 8); after the 4th pair of a BFP16 block, write the block to LDS
    // (bf16, [row][k], pitch PA).
    template <int set, int i, int t>
    ATB_DEV void decode_pair(char *a_dst)
    {
        if constexpr (t % 4 == 0) shift = (int)((a_expo[set][i] >> (8 * (t / 4))) & 0xFFu) - 133;
        const int w = a_mant[set][i][t / 2];
        const float f0 = ldexpf(mant_to_float(w, (t % 2) * 2), shift);
        const float f1 = ldexpf(mant_to_float(w, (t % 2) * 2 + 1), shift);
        union { bf16x2 v; unsigned u; } pk;
        pk.v = bf16x2{(__bf16)f0, (__bf16)f1};
        dec[t % 4] = pk.u;
        if constexpr (t % 4 == 3) {
            char *dst = a_dst + (a_row + i * (S::NT / S::A_CPR)) * S::PA + a_q * (S::ACE * 2) + (t / 4) * 16;
            *reinterpret_cast<intx4 *>(dst) = intx4{(int)dec[0], (int)dec[1], (int)dec[2], (int)dec[3]};
        }
    }

    template <int i>
    ATB_DEV void store_b_chunk(char *b_dst)
    {
        *reinterpret_cast<intx4 *>(b_dst + (b_row + i * (S::NT / S::B_CPR)) * S::PB + b_c * 16) = b_raw[i];
    }

    template <int set, int j = 0>
    ATB_DEV void store_a_all(char *a_dst)
    {
        if constexpr (j < S::NPAIR) {
            decode_pair<set, j / (S::ACE / 2), j % (S::ACE / 2)>(a_dst);
            store_a_all<set, j + 1>(a_dst);
        }
    }

    template <int i = 0>
    ATB_DEV void store_b_all(char *b_dst)
    {
        if constexpr (i < S::B_PER_THREAD) {
            store_b_chunk<i>(b_dst);
            store_b_all<i + 1>(b_dst);
        }
    }

    // ---- LDS -> registers ----------------------------------------------------------------
    // The wave's B fragments for one K-step: bfrag[ks][nt] holds, per lane l, column
    // (wn*NTW + nt)*32 + l%32 and k = ks*16 + 8*(l/32) .. +7.  B sits row-major ([k][n]) in LDS;
    // ds_read_b64_tr_b16 transposes on the way out: within each group of 16 lanes, lane i addresses
    // 4 consecutive columns of row i/4, and lane j receives column j of those 4 rows.
    ATB_DEV void read_b_frags(const char *b_src)
    {
        const int blk = lane >> 4, j = lane & 15;
        const char *base = b_src + (8 * (blk >> 1) + (j >> 2)) * S::PB +
                           (wn * S::NTW * 32 + 16 * (blk & 1) + 4 * (j & 3)) * 2;
#pragma unroll
        for (int ks = 0; ks < S::KS; ++ks) {
#pragma unroll
            for (int nt = 0; nt < S::NTW; ++nt) {
                const char *src = base + ks * 16 * S::PB + nt * 64;
                typedef __attribute__((address_space(3))) shortx4 lds_shortx4;
                union { shortx4 s[2]; bf16x8 b; } u;
                u.s[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_shortx4 *)(src));
                u.s[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_shortx4 *)(src + 4 * S::PB));
                bfrag[ks][nt] = u.b;
            }
        }
    }

    // A fragment (band il of the sub-tile, k-slice ks): lane l reads row l%32, k = ks*16 + 8*(l/32) .. +7.
    // Bands of the C tile are dealt round-robin to the wave rows: band il*WM + wm of the sub-tile.
    template <int il, int ks>
    ATB_DEV void read_a_frag(const char *a_src)
    {
        const char *src = a_src + ((il * S::WM + wm) * 32 + (lane & 31)) * S::PA + (lane >> 5) * 16 + ks * 32;
        afrag[il % 2][ks] = *reinterpret_cast<const bf16x8 *>(src);
    }

    // ---- one microkernel, software-pipelined by hand ---------------------------------------
    // Side work j of phase s: decode + LDS write of the next A sub-tile, then (last phase of the
    // K-step) the LDS writes of the next B tile.
    template <int s, int j>
    ATB_DEV void side(char *a_dst, char *b_dst)
    {
        if constexpr (j < S::NPAIR) {
            decode_pair<0, j / (S::ACE / 2), j % (S::ACE / 2)>(a_dst);
        } else {
            store_b_chunk<j - S::NPAIR>(b_dst);
        }
    }

    template <int s, int j, int jend>
    ATB_DEV void side_range(char *a_dst, char *b_dst)
    {
        if constexpr (j < jend) {
            side<s, j>(a_dst, b_dst);
            side_range<s, j + 1, jend>(a_dst, b_dst);
        }
    }

    // Slot m: one MFMA, then its share of the side work and (after the last column band of a
    // k-slice) the A fragment of the same k-slice of the next band.  The fences pin this order, so
    // the VALU decode and the LDS traffic issue in the shadow of the 8-pass MFMA.
    template <int s, int m>
    ATB_DEV void slots(const char *a_src, char *a_dst, char *b_dst)
    {
        if constexpr (m < S::NM) {
            constexpr int il = m / (S::KS * S::NTW), ks = (m / S::NTW) % S::KS, nt = m % S::NTW;
            constexpr int local = (s * S::SMT) / S::WM + il;      // accumulator band of this wave
            constexpr int nside = S::NPAIR + ((s + 1 == S::RHO) ? S::B_PER_THREAD : 0);
            acc[local][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfrag[ks][nt], afrag[il % 2][ks],
                                                                    acc[local][nt], 0, 0, 0);
            ATB_FENCE();
            side_range<s, (m * nside) / S::NM, ((m + 1) * nside) / S::NM>(a_dst, b_dst);
            if constexpr (nt == S::NTW - 1 && il + 1 < S::PER) read_a_frag<il + 1, ks>(a_src);
            ATB_FENCE();
            slots<s, m + 1>(a_src, a_dst, b_dst);
        }
    }

    template <int ks = 0>
    ATB_DEV void read_first_band(const char *a_src)
    {
        if constexpr (ks < S::KS) {
            read_a_frag<0, ks>(a_src);
            read_first_band<ks + 1>(a_src);
        }
    }

    // The raw A sub-tiles in flight form a queue of PF register sets: set 0 is decoded next, a new
    // fetch goes into set PF-1.
    ATB_DEV void shift_a_queue()
    {
#pragma unroll
        for (int q = 0; q + 1 < S::PF; ++q)
#pragma unroll
            for (int i = 0; i < S::A_PER_THREAD; ++i) {
                a_mant[q][i] = a_mant[q + 1][i];
                a_expo[q][i] = a_expo[q + 1][i];
            }
    }

    // Phase s of K-step kt: microkernel on sub-tile s, while sub-tile s+1 is decoded into the other
    // LDS buffer and sub-tile s+PF is fetched from memory.  Sub-tile g = kt*RHO + s sits in LDS
    // buffer g % 2.
    template <int s>
    ATB_DEV void phases(int kt)
    {
        if constexpr (s < S::RHO) {
            const int k0 = kt * S::T_K;
            const int cur = (S::RHO % 2 == 0) ? (s & 1) : ((kt + s) & 1);
            {
                constexpr int sf = (s + S::PF) % S::RHO, kf = (s + S::PF) / S::RHO;
                load_a(m0 + sf * S::T_MA, k0 + kf * S::T_K);
            }
            if constexpr (s == 0) load_b(k0 + S::T_K);
            ATB_FENCE();                 // keep the memory requests ahead of everything else
            const char *a_src = cur ? a_lds[1] : a_lds[0];
            char *a_dst = cur ? a_lds[0] : a_lds[1];
            char *b_dst = (kt & 1) ? b_lds[0] : b_lds[1];
            read_first_band(a_src);
            ATB_FENCE();
            slots<s, 0>(a_src, a_dst, b_dst);
            shift_a_queue();
            __syncthreads();             // the "kernel switch" of the ATB nest
            phases<s + 1>(kt);
        }
    }

    template <int g = 0>
    ATB_DEV void prologue_loads()
    {
        if constexpr (g < S::PF) {
            load_a<g>(m0 + (g % S::RHO) * S::T_MA, (g / S::RHO) * S::T_K);
            prologue_loads<g + 1>();
        }
    }

    ATB_DEV void run()
    {
        // prologue: first B tile, the first PF A sub-tiles into registers, sub-tile 0 into LDS
        load_b(0);
        prologue_loads();
        store_b_all(b_lds[0]);
        store_a_all<0>(a_lds[0]);
        shift_a_queue();
        __syncthreads();

        const int KT = (p.K + S::T_K - 1) / S::T_K;
        for (int kt = 0; kt < KT; ++kt) {
            read_b_frags((kt & 1) ? b_lds[1] : b_lds[0]);
            phases<0>(kt);
        }
        store_c();
    }

    // epilogue: fp32 -> bf16 (round to nearest even) and store, once per tile.  Lane l of band
    // (a, b) holds row l%32 and columns 8*g + 4*(l/32) + 0..3 for g = 0..3.
    ATB_DEV void store_c()
    {
        const bool st_vec = (p.N % 4) == 0;
#pragma unroll
        for (int a = 0; a < S::MTW; ++a) {
            const int m = m0 + (a * S::WM + wm) * 32 + (lane & 31);
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
};

template <class S, bool VEC>
__global__ void __launch_bounds__(S::NT) atb_gemm_kernel(const GemmParams p)
{
    __shared__ __attribute__((aligned(16))) char lds[S::LDS_BYTES];

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

    TileKernel<S, VEC> t(p, lds, tm * S::T_MC, tn * S::T_N);
    t.run();
}

template <class S>
hipError_t launch_instance(const GemmParams &p, hipStream_t stream)
{
    const int total = p.tiles_m * p.tiles_n;
    const int per_xcd = (total + 7) / 8;
    if ((p.N % 8) == 0)
        hipLaunchKernelGGL((atb_gemm_kernel<S, true>), dim3(per_xcd * 8), dim3(S::NT), 0, stream, p);
    else
        hipLaunchKernelGGL((atb_gemm_kernel<S, false>), dim3(per_xcd * 8), dim3(S::NT), 0, stream, p);
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

const Instance g_instances[] = {
    // T_MC = T_N = 256, T_K = 64: the sweep over rho = 1, 2, 4, 8
    make_instance<Shape<256, 256, 64, 256, 2, 2, 2>>(),
    make_instance<Shape<128, 256, 64, 256, 2, 2, 2>>(),
    make_instance<Shape<64, 256, 64, 256, 2, 2, 2>>(),
    make_instance<Shape<32, 256, 64, 256, 1, 4, 4>>(),
    // small tiles for small problems
    make_instance<Shape<64, 64, 64, 64, 2, 2, 1>>(),
    make_instance<Shape<32, 64, 64, 64, 1, 2, 2>>(),
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
