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
//   * one workgroup barrier per sub-tile is the "kernel switch" of Sec. 5;
//   * workgroups of 8 waves (two per SIMD) split the staging by kind: waves 0-3 stage A, waves 4-7
//     stage B (see TileKernel); the grid of the 256 x 256 tiles is persistent (see tile_loop).
//     Smaller tiles have a grid of 4 or 2 multiplying waves plus as many helper waves that do the staging.
// T_MA == T_MC is the symmetric baseline: same code, one sub-tile per K-step.
// B may also arrive as BFP16 (as B^T, blocks along K) and C may be written as BFP16 (Sec. 6.1's
// all-BFP16 storage); see the BBFP / CBFP template flags of TileKernel.
//
// MFMA: v_mfma_f32_16x16x32_bf16 or v_mfma_f32_32x32x16_bf16 (Shape::MB = 16 or 32 says which and why).
// Operand lane layout: lane l supplies row (l % MB) of its operand and the 8 consecutive k values
// 8*(l/MB) .. +7, which for the A operand is exactly one BFP16 block.  The B fragment is passed as
// the first operand and the A fragment as the second, so a lane of the result holds one row m
// (= l % MB) and groups of 4 consecutive columns (n = 8*g + 4*(l/MB) + 0..3) -> 8-byte bf16 stores.
#include <algorithm>
#include <mutex>

#include "atb_internal.h"

namespace atb {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef short shortx4 __attribute__((ext_vector_type(4)));

#define ATB_DEV __device__ __forceinline__

// Sign-extended byte `byte` of word w as float (one v_cvt_f32_i32 with a byte select).
ATB_DEV float mant_to_float(int w, int byte) { return (float)(int)(signed char)(w >> (8 * byte)); }

template <int T_MA_, int T_MC_, int T_K_, int T_N_, int WM_, int WN_, int PF_, int AB_ = 2, int AO_ = -1, int BO_ = 0, int KU_ = 2, int NB_ = 2, int HW_ = 0, int SKEW_ = 0, int MB_ = 0, int OCC_ = 1, bool ADMA_ = false>
struct Shape {
    static constexpr int T_MA = T_MA_, T_MC = T_MC_, T_K = T_K_, T_N = T_N_, WM = WM_, WN = WN_;
    static constexpr int PF = PF_;                // A sub-tiles fetched this many phases ahead of their use
    static constexpr int KU = KU_;                // K-steps per iteration of the (unrolled) K loop: every buffer and register-set index is static
    // A LDS buffers.  2: sub-tile g+1 is decoded while sub-tile g is multiplied, and each microkernel
    // starts by reading its first fragments after the switch barrier.  4: the small A sub-tiles of
    // ATB leave room for a deeper ring: sub-tile g+2 is decoded while g is multiplied, so sub-tile
    // g+1 is already complete and its first fragments are read before the barrier, which takes the
    // LDS latency out of every switch.
    static constexpr int AB = AB_;
    // B LDS buffers.  The tile of K-step kt + NB is requested during K-step kt into the buffer that the
    // tile of K-step kt has just left.  2 is enough when the tiles are large and many workgroups keep the
    // memory busy; problems with one row of C tiles have fewer workgroups than CUs and live on the bytes each
    // workgroup keeps in flight, so their instances use a ring of 3 or more (indexed at run time).
    static constexpr int NB = NB_;
    static constexpr int DA = (AB_ == 4) ? 2 : 1; // decode runs this many sub-tiles ahead
    static constexpr int CW = WM * WN;            // waves that multiply: a WM x WN grid over the C tile
    // Helper waves.  Small tiles have few wave tiles (a 64 x 64 tile at T_MA = 32 feeds a 1 x 2 grid), and a
    // wave that stages, decodes and multiplies issues all of it in order.  With HW > 0 the staging (requests,
    // decode, LDS stores) moves to HW extra waves on the CU's other SIMDs and the CW waves only multiply.
    static constexpr int HW = HW_;
    static constexpr int NT = (CW + HW) * 64;     // threads
    // Staging is dealt out in slabs of NTS chunks (one chunk per thread of a group of NTS threads).
    // 8-wave workgroups run two waves per SIMD and form two groups, waves 0-3 and 4-7; the first
    // group stages A slabs [0, AO) and B slabs [0, BO) of every (sub-)tile, the second the rest.
    static constexpr int NTS = (HW > 0) ? HW * 64 : (CW == 8) ? 256 : CW * 64;
    static constexpr int RHO = T_MC / T_MA;
    static constexpr int MT = T_MC / 32;          // 32-row bands in the C tile
    static constexpr int SMT = T_MA / 32;         // bands per A sub-tile
    static constexpr int MTW = MT / WM;           // bands per wave
    static constexpr int NTW = T_N / 32 / WN;     // 32-column bands per wave
    // The MFMA.  gfx950 has two bf16 forms of the same peak rate: 32 x 32 x 16 (rows x columns x k per instruction)
    // and 16 x 16 x 32.  The first needs half as many operand registers and instructions per flop; the second is the
    // cheaper one in power, and this chip is power-limited: an MFMA-only loop on random bf16 operands sustains
    // 2.07 PFLOP/s with 16 x 16 x 32 against 1.83 with 32 x 32 x 16.  MB = 16 where two waves of the workgroup share a
    // SIMD (the other wave's instructions fill the gaps between the short MFMAs: +2 to +6 % on 8192^3, box to box),
    // MB = 32 where a SIMD has one multiplying wave per workgroup, whose single instruction stream cannot issue twice
    // as many MFMAs and their operand reads without gaps (rho = 8: 10 % slower with MB = 16), unless the instance
    // says otherwise.  The two forms give bit-equal results.
    // A 32-row band of A is HB row blocks of MB rows.
    static constexpr int MB = MB_ ? MB_ : (WM * WN == 8 ? 16 : 32);
    // Waves per SIMD that the kernel is compiled for (the second argument of __launch_bounds__: the register
    // allocator then stays within 512 / OCC registers, spilling if it must).  Set where a few registers too many
    // would cost a whole workgroup per CU.
    static constexpr int OCC = OCC_;
    static constexpr int KM = 512 / MB;           // k per MFMA
    static constexpr int HB = 32 / MB;            // row blocks per band
    static constexpr int NC = T_N / MB / WN;      // column blocks per wave
    static constexpr int KS = T_K / KM;           // MFMA k-slices per K-step
    static constexpr int ACC = MB * MB / 64;      // accumulator registers per block
    // Order of a band's MFMAs.  KIN: the k-slices of one accumulator block follow each other (then the column blocks,
    // then the row blocks), so that an MFMA adds to the result of the one before it; otherwise the column blocks that
    // share an A fragment follow each other.  With two waves per SIMD the other wave's MFMAs fill the wait for the
    // dependent one, and the chained order measured 0.3 to 1.4 % faster on 8192^3 for the 256 x 256 tile at rho = 1
    // and 2 (three boxes); level or up to 1 % slower at rho = 4 and for the 128-row tiles, which keep the other order.
    static constexpr bool KIN = (WM * WN == 8 && T_MC == 256 && T_MA >= 128);
    static constexpr int PER = SMT / WM;          // bands of one sub-tile per wave row
    // LDS pitches in bytes, and how the rows of a tile staged as [row][k] (A; B^T in BFP16) keep out of each other's
    // banks.  The LDS serves a 16-byte read of a wave in four passes of 16 lanes -- lanes 0-3, 12-15, 20-27; lanes
    // 4-11, 16-19, 28-31; and the same plus 32 -- and a 16-byte store in eight passes of 8 consecutive lanes that
    // must differ in address bits 4-6 (measured lane pair by lane pair with the bank-conflict counter).
    // MB = 32 (a lane reads row l % 32, chunk l / 32): rows padded by 16 bytes; a pass then sees 16 rows whose
    // starts are 36 banks apart.  MB = 16 (row l % 16, chunk l / 16: a pass mixes two chunk columns) would lose four
    // cycles per read to conflicts with that pitch.  ASWZ: no padding; chunk c of row r sits at position c ^ (r % 8)
    // of its 128-byte row instead, which is conflict-free for these reads and for the staging stores (a thread's 32
    // or 64 bytes of a row, four or two threads per row) -- found by searching the XOR swizzles that are linear in
    // the row's bits.  It also saves 16 bytes per row.
    static constexpr bool ASWZ = (MB == 16 && T_K == 64);
    // Uneven deal of the C tile's 32-row bands between the two wave groups of an 8-wave workgroup: the group that
    // decodes A (waves 0-3) multiplies SKEW bands fewer per C tile than its even share and the other group SKEW more,
    // so that the decoding waves' longer instruction stream and the other waves' shorter one end a phase together.
    // The wave grid is then laid out with the wave row equal to the group (see TileKernel).
    static constexpr int SKEW = SKEW_;
    static constexpr int PA = ASWZ ? T_K * 2 : T_K * 2 + 16;
    static constexpr int PBF = PA;                // B^T in BFP16 is staged like A
    static constexpr int PB = T_N * 2;            // B rows are not padded: an XOR swizzle of the 16-byte chunks avoids the bank conflicts
    static constexpr int A_BYTES = T_MA * PA;
    static constexpr int B_BYTES = T_K * PB;
    // ADMA: the A sub-tiles reach the CU as B does, requested by the second wave group straight into LDS -- as they
    // lie in memory, 64 mantissa bytes and 8 exponent bytes per row (the K-panel-major planes make a sub-tile's share
    // of a K-step one contiguous run of each) -- into a ring of NR raw buffers; the decoding waves read their chunks
    // from there instead of from memory, and issue no memory instruction at all.  The ring is what ATB's smaller A
    // buffers pay for: 36 KiB at T_MA = 128, which does not fit next to a symmetric 256-row tile (its ring would be
    // 72 KiB; even two raw buffers, 36 KiB, put it at 164 KiB).  Measured: the decoding waves wait less, the
    // throughput does not change (the bytes cost the same whichever way they come in); an experiment, off by default.
    static constexpr bool ADMA = ADMA_;
    static constexpr int NR = 4;                                   // raw buffers: sub-tile g uses buffer g % NR
    static constexpr int RAW_BYTES = T_MA * (kPanelK + kPanelK / 8);
    static constexpr int RAW_RING = ADMA ? NR * RAW_BYTES : 0;
    static constexpr int LDS_BYTES = AB * A_BYTES + NB * B_BYTES + RAW_RING;
    // B given as BFP16 (B^T, N x K, blocks along K): the tile is staged like A, [n][k] with pitch PA
    static constexpr int BT_BYTES = T_N * PBF;
    static constexpr int LDS_BYTES_BT = AB * A_BYTES + 2 * BT_BYTES;
    static constexpr int BT_SLABS = T_N * T_K / 16 / NTS;      // 16-mantissa chunks of the tile per staging thread
    // staging work per thread: A in chunks of ACE mantissas (ACE/8 BFP16 blocks), B in chunks of 8 bf16
    static constexpr int ACE = (T_MA * T_K / NTS >= 16) ? 16 : 8;
    static constexpr int A_CHUNKS = T_MA * T_K / ACE;
    static constexpr int A_SLABS = A_CHUNKS / NTS;
    static constexpr int AO = (AO_ < 0) ? A_SLABS : AO_;   // default: the first group stages all of A ...
    static constexpr int A_CPR = T_K / ACE;       // chunks per A row
    static constexpr int B_CHUNKS = T_K * (T_N / 8);
    static constexpr int B_SLABS = B_CHUNKS / NTS;
    static constexpr int BO = BO_;                          // ... and the second all of B
    static constexpr int B_CPR = T_N / 8;         // 16-byte chunks per B row
    // B swizzle: chunk c of row k sits at chunk position c ^ b_swz(k) of its row, so that the pieces of different
    // rows that one transposing read touches fall into different LDS banks.
    // MB = 32: per 32 lanes, 4 rows x 2 neighbouring 32-byte pieces; k mod 4 goes into bits 2-3 of the position and the
    // 8 pieces cover 256 consecutive bytes, i.e. every bank once.  Narrow tiles (rows of 8 chunks) can only afford
    // bits 1-2, which keeps 16 lanes conflict-free.
    // MB = 16: per 32 lanes, the rows k0 .. k0+3 and k0+8 .. k0+11 of one 16-column block, 32 bytes of each.  Rows
    // of 16 or more chunks (a multiple of 256 bytes, so all rows start in the same bank): bits 2-3 of the position
    // from k mod 4, bit 1 from bit 3 of k.  Rows of 8 chunks (128 bytes: odd rows start half way round the banks,
    // which separates k and k+1): bit 1 from bit 1 of k, bit 2 from bit 3 of k.
    static constexpr bool WIDE = (T_N / 8 >= 16);
    static constexpr int b_swz(int k)
    {
        if (MB == 32) return (k & 3) << (WIDE ? 2 : 1);
        return WIDE ? (((k & 3) << 2) | (((k >> 3) & 1) << 1)) : ((((k >> 1) & 1) << 1) | (((k >> 3) & 1) << 2));
    }
    static constexpr int NBASE = (NC < 4) ? NC : 4;     // distinct per-lane read bases: the swizzle permutes groups of four column blocks
    static_assert(MB == 32 || NC <= 4, "MB = 16: the B swizzle permutes the wave's (at most four) column blocks");
    static_assert(T_MC % T_MA == 0, "rho must be an integer");
    static_assert(MB == 32 || ASWZ, "MB = 16 reads need the swizzled rows, which are written for rows of 8 chunks (T_K = 64)");
    static_assert(NB >= 2, "the B tile being multiplied and the one being fetched");
    static_assert(KU % 2 == 0 && PF >= 2 && (KU * RHO) % PF == 0, "prefetch distance: at least 2 (fetch and decode overlap), dividing the sub-tiles of one loop iteration");
    static_assert(AB == 2 || (AB == 4 && PF >= 3 && (KU * RHO) % 4 == 0), "4 A buffers need a fetch distance of 3 or more and must divide the sub-tiles of one loop iteration");
    static_assert(T_K % 64 == 0, "a K-step is a whole number of 64-wide panels of the BFP16 layout");
    static_assert(MB == 16 || MB == 32, "v_mfma_f32_16x16x32_bf16 or v_mfma_f32_32x32x16_bf16");
    static_assert(T_MA % 32 == 0 && T_N % (32 * WN) == 0 && T_K % 32 == 0, "bands of 32 rows and columns, MFMA k-slices of 16 or 32");
    static_assert(MT % WM == 0 && SMT % WM == 0, "every sub-tile must feed every wave row equally");
    static_assert(A_CHUNKS % NTS == 0 && NTS % A_CPR == 0, "A staging must split evenly over the threads");
    static_assert(B_CHUNKS % NTS == 0 && NTS % B_CPR == 0, "B staging must split evenly over the threads");
    static_assert(AO >= 0 && AO <= A_SLABS && BO >= 0 && BO <= B_SLABS, "staging split");
    static_assert(B_CPR >= 8, "the B swizzle needs 8 chunks per row");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget of a gfx950 CU");
    static_assert(!ADMA || (WM * WN == 8 && HW == 0 && T_K == kPanelK && T_MA == 128 && AB == 2 && PF == 2 && (KU * (T_MC / T_MA)) % NR == 0),
                  "raw A staging: two wave groups, one K-panel per K-step, one KiB of mantissas per wave and request, static ring indices");
    static_assert((MTW + SKEW) * HB * NC * ACC <= 256, "C tile must fit the accumulator registers");
    static_assert(SKEW == 0 || (CW == 8 && WM == 2 && HW == 0 && AB == 2 && SKEW < MTW), "the uneven deal is between the two wave groups of a 2 x 4 grid");
};

typedef int intx4 __attribute__((ext_vector_type(4)));
typedef int intx2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// Buffer descriptors (V#) of the three inputs.  A load whose byte offset lies outside
// [0, num_records) returns zero without touching memory, which is what masks the edges.
struct Rsrc {
    __amdgpu_buffer_rsrc_t am, ae, b, bm, be;
    intx4 b_words;      // the B descriptor once more as four dwords, for the hand-issued requests of the symmetric instances
    intx4 am_words, ae_words;   // likewise the A descriptors, for the raw requests (ADMA)
};

constexpr int kRsrcFlags = 0x00020000;           // raw buffer, 32-bit data format

#define ATB_FENCE() __builtin_amdgcn_sched_barrier(0)

// MFMAs issued back to back per slot of the hand-made pipeline (see TileKernel::slots)
#ifndef ATB_MFMA_GROUP
#define ATB_MFMA_GROUP 1
#endif

// Origin of the t-th tile of this workgroup's XCD (false past the end of the walk).  Workgroups
// are dealt round-robin to the 8 XCDs (each with its own L2); XCD x owns the contiguous run of
// tiles [x * per_xcd, (x + 1) * per_xcd), walked in bands of group_m tile rows so that the
// workgroups resident on one XCD share few distinct A row panels and B column panels.
template <class S>
ATB_DEV bool tile_origin(const GemmParams &p, int t, int &tm0, int &tn0)
{
    const int total = p.tiles_m * p.tiles_n;
    const int per_xcd = (total + 7) / 8;
    const int logical = (int)(blockIdx.x % 8) * per_xcd + t;
    if (t >= per_xcd || logical >= total) return false;
    const int band_sz = p.group_m * p.tiles_n;
    const int band = logical / band_sz, in_band = logical % band_sz;
    const int rows_here = min(p.group_m, p.tiles_m - band * p.group_m);
    tm0 = (band * p.group_m + in_band % rows_here) * S::T_MC;
    tn0 = (in_band / rows_here) * S::T_N;
    return true;
}

// Bands of the C tile per wave.  Even deal: band il * WM + wm of every sub-tile, PER per sub-tile.  Uneven deal
// (Shape::SKEW, only where the first wave group decodes and the second does not): the first group's waves form wave
// row 0 and take the first per(s) bands of sub-tile s, the second group's the rest.
template <class S, int ROLE, bool VEC, bool BBFP>
struct BandDeal {
    static constexpr bool SKEWED = S::SKEW > 0 && (ROLE == 1 || ROLE == 2) && VEC && !BBFP;   // (the odd-N path has no registers to spare for it)
    static constexpr int moved(int s) { return SKEWED ? (S::SKEW * (s + 1)) / S::RHO - (S::SKEW * s) / S::RHO : 0; }   // bands of sub-tile s that change hands
    static constexpr int per(int s) { return ROLE == 1 ? S::PER - moved(s) : ROLE == 2 ? S::PER + moved(s) : S::PER; }
    static constexpr int first_local(int s) { int n = 0; for (int t = 0; t < s; ++t) n += per(t); return n; }         // accumulator band of the wave's first band of sub-tile s
    // band of sub-tile s that this wave's il-th band is, not counting the wave row's own offset in the even deal
    static constexpr int band(int s, int il) { return SKEWED ? (ROLE == 1 ? il : S::PER - moved(s) + il) : il * S::WM; }
};

// The per-workgroup state of one C tile.  Everything is indexed with compile-time constants after
// inlining, so the arrays live in registers (acc in AccVGPRs).
//
// Time line (g = kt*RHO + s numbers the A sub-tiles):
//   A sub-tile g   : fetched from memory in phase g-PF into register set g % PF, decoded into LDS
//                    buffer g % 2 during phase g-1, consumed by the microkernel of phase g.
//   B tile kt      : requested in the first phase of K-step kt-2 straight into LDS buffer kt % 2
//                    (odd N: into registers, written to LDS in the last phase of K-step kt-2),
//                    awaited before the last barrier that precedes the last band of K-step kt-1,
//                    read into the waves' fragment registers during that band (each fragment
//                    right after its last use), consumed in K-step kt.
// The K loop is unrolled by two so that every buffer and register-set index is a constant.
// The time line does not stop at the end of a tile: when a request stream has asked for the last
// K-step of its tile it moves on to the first K-step of the workgroup's next tile (open_a, open_b),
// so K-step 0 of that tile finds its operands staged exactly as any other K-step does.
//
// Staging roles.  ROLE 0: every wave stages its share of A and of B.  Workgroups of 8 waves run two
// waves per SIMD, and the SIMD's arbiter prefers the older one (measured: with equal work the first
// four waves finish a microkernel a third earlier and then idle at the barrier while the others run
// on alone, slowly).  There the staging work is split by kind instead of evenly: ROLE 1 (waves 0-3)
// fetches, decodes and stores all of A, ROLE 2 (waves 4-7) requests all of B, which costs it a few
// memory instructions and no arithmetic, so both waves of a SIMD reach the barrier together.
// Tiles with fewer than eight wave tiles (Shape::HW > 0) use the same idea the other way round: ROLE 4
// (the WM x WN grid of waves) only reads fragments and multiplies, ROLE 3 (HW helper waves) stages all of
// A and B and multiplies nothing; both execute the same sequence of barriers.
//
// Storage formats (Sec. 6.1 lists the paper's precision configurations).  BBFP: B arrives as BFP16,
// given as B^T (N x K, blocks along K, the same layout as A); its tile is fetched into registers,
// decoded and stored to LDS as [n][k] like an A sub-tile -- by the second wave group, while the first
// does the same for A -- and its fragments are plain 16-byte LDS reads.  Tile kt is fetched in the
// first phase of K-step kt-3, decoded during K-step kt-2, read into fragment registers in the last
// band of K-step kt-1.  CBFP: the epilogue quantises C to BFP16 in blocks of 8 along N.
// BTR: B arrives as bf16 but transposed, B^T (N x K, the K index contiguous: the layout in which frameworks keep the
// weight of a linear layer).  Its tile still goes global -> LDS directly, now as [n][k] rows of 2 T_K bytes whose
// 16-byte chunks are XOR-swizzled by (n / 2) mod 8, and an MFMA fragment is ONE plain 16-byte LDS read per lane
// instead of two transposing 8-byte reads (half the LDS read instructions for B).
template <class S, bool VEC, int ROLE, bool BBFP = false, bool CBFP = false, bool SK = false, bool BTR = false>
struct TileKernel {
    static constexpr int NTS = S::NTS, ACE = S::ACE, A_CPR = S::A_CPR;
    static constexpr int AO = BBFP ? S::A_SLABS : S::AO;                                 // with B in BFP16 the second group has its hands full
    static constexpr bool COMPUTE = (ROLE != 3);                                         // ROLE 3: helper waves (stage everything, multiply nothing); ROLE 4: their partners (multiply only)
    static constexpr int A_FIRST = (ROLE == 2) ? AO : 0;                                 // first A slab of this wave group
    static constexpr int APT = (ROLE == 0 || ROLE == 3) ? S::A_SLABS : (ROLE == 1) ? AO : (ROLE == 2) ? S::A_SLABS - AO : 0;   // A chunks per thread per sub-tile
    static constexpr int NPAIR = APT * ACE / 2;                                          // mantissa pairs per thread per sub-tile
    // A thread with two 16-mantissa chunks takes them side by side in one row (32 consecutive k): their
    // four exponent bytes are one aligned dword, so one exponent request serves both chunks.
    // Raw A staging through LDS (Shape::ADMA): ROLE 2 requests the sub-tiles, ROLE 1 reads its chunks from the raw ring.
    static constexpr bool ADMA_ON = S::ADMA && VEC && !BBFP && !SK && (ROLE == 1 || ROLE == 2);
    static constexpr int RQM = S::T_MA / 64;                 // 1 KiB mantissa requests per wave of the group and sub-tile
    static constexpr int RQ = (ADMA_ON && ROLE == 2) ? RQM + 1 : 0;   // ... plus one 256-byte request for the exponents
    static constexpr int RAW_LEAD = S::PF + 2;               // sub-tile x is requested in phase x - RAW_LEAD, complete one phase later, read in phase x - PF
    static constexpr bool PAIRK = (APT == 2 && ACE == 16 && A_FIRST == 0 && S::T_K == 64 && !ADMA_ON);
    static constexpr int A_VMEM = PAIRK ? 3 : APT * 2;       // memory requests per thread and A sub-tile
    // Rows >= M of an edge tile only feed rows of C that are never stored.  SK is the variant of the kernel
    // for tiles at least half of whose rows lie beyond M (skinny problems, where that is most of the VALU
    // work): it decodes block by block and skips, wave by wave, the chunks without a row below M.  (Their
    // requests are still issued: the explicit vmcnt waits count requests.)
    static_assert(!SK || (S::RHO * APT <= 32 && !BBFP), "one liveness bit per chunk of the tile");
    static constexpr int B_FIRST = (ROLE == 2) ? S::BO : 0;
    static constexpr int BPT = BBFP ? 0 : (ROLE == 0 || ROLE == 3) ? S::B_SLABS : (ROLE == 1) ? S::BO : (ROLE == 2) ? S::B_SLABS - S::BO : 0;   // bf16 B chunks per thread per tile
    static constexpr int BTPT = !BBFP ? 0 : (ROLE == 1 || ROLE == 4) ? 0 : S::BT_SLABS;               // BFP16 B chunks (16 mantissas) per thread per tile
    static constexpr int NPAIR_B = BTPT * 8;                                             // B mantissa pairs per thread per tile
    static constexpr int NSTEP_A = NPAIR == 0 ? 0 : SK ? NPAIR / 4 : NPAIR + 2;          // decode items per phase (A sub-tile): pipeline steps, or blocks
    static constexpr int NSTEP_B = NPAIR_B > 0 ? NPAIR_B / S::RHO + 2 : 0;               // ... and for this phase's share of the B tile
    static constexpr bool ASM_DMA = VEC && !BBFP && S::RHO <= 2 && APT == 0 && BPT > 0;   // B requests issued by hand, see load_b_chunk
    // a wave group that issues requests by hand issues no other loads: the compiler's own vmcnt waits (for loads it
    // knows of) would otherwise count the hand-issued requests as well, and its built-in LDS-direct loads use M0 too
    static_assert(!ASM_DMA || (APT == 0 && BTPT == 0 && VEC && !BBFP), "hand-issued B requests only in wave groups without compiler-visible loads");
    static constexpr int APTN = APT > 0 ? APT : 1, BPTN = BPT > 0 ? BPT : 1, BTPTN = BTPT > 0 ? BTPT : 1;   // array extents
    static constexpr int B_BYTES = BBFP ? S::BT_BYTES : S::B_BYTES;
    static_assert(!BBFP || (NPAIR_B % S::RHO == 0 && S::T_K % 16 == 0 && (S::T_N * S::T_K / 16) % NTS == 0), "BFP16 B staging must split evenly");
    static_assert(!BBFP || S::LDS_BYTES_BT <= 160 * 1024, "LDS budget of a gfx950 CU (the BFP16 B path always has two buffers)");
    static_assert((ROLE == 0) == (S::CW != 8 && S::HW == 0) && (ROLE >= 3) == (S::HW > 0), "two staging groups exactly when two waves share a SIMD; helper roles exactly with helper waves");
    static_assert(!BTR || (VEC && !BBFP && !SK && S::T_K == 64), "the transposed-B path: bf16 B^T, K-steps of 64 (8 chunks per LDS row, swizzled over 8 row pairs)");
    static constexpr int PBT = S::T_K * 2;                                                // LDS pitch of a B^T tile row
    typedef BandDeal<S, ROLE, VEC, BBFP> D;
    static constexpr bool SKEWED = D::SKEWED;
    static constexpr int MTW = D::first_local(S::RHO);                                    // accumulator bands of this wave
    static constexpr int per(int s) { return D::per(s); }
    static constexpr int first_local(int s) { return D::first_local(s); }
    static constexpr int band(int s, int il) { return D::band(s, il); }
    static constexpr int nm(int s) { return D::per(s) * S::HB * S::KS * S::NC; }              // MFMAs of this wave in phase s
    static constexpr int bands_before(int g) { return (g / S::RHO) * MTW + D::first_local(g % S::RHO); }   // running band count at sub-tile g of the loop body

    const GemmParams &p;
    Rsrc rs;
    int tid, lane, wm, wn;
    // The workgroup walks its C tiles t_first, t_first + t_stride, ... (see tile_at) as one unbroken
    // pipeline: the requests for A and for B run ahead of the arithmetic by fixed numbers of K-steps,
    // across tile boundaries too, so each of the three streams keeps its own position in the walk.
    int t_stride, kt_steps;            // kt_steps: K-steps per tile, rounded up to a whole loop body
    int c_t, m0, n0;                   // the tile being accumulated (and stored by the epilogue)
    int a_t, a_m0, a_steps;            // A requests: tile, the row origin the offsets are based on, K-steps left to request
    int b_t, b_n0, b_steps;            // B requests: likewise with the column origin
    // LDS byte addresses of this thread's staging writes and fragment reads, per buffer
    char *a_wr[S::AB], *b_wr[2];
    const char *a_rdk[S::KS];          // ASWZ: this lane's fragment read address per k-slice, in A buffer 0, band 0
    int a_d[4];                        // ASWZ: byte offset of 16-byte piece p of this thread's run of a row from its piece 0 (a_wr points at piece 0)
    static constexpr int NRD = BTR ? S::KS : S::NBASE;
    const char *a_rd[S::AB], *b_rd[2][NRD];       // b_rd[buffer][column band mod 4]; transposed B: b_rd[buffer][k-slice]
    char *b_req[2];                    // LDS byte address of this wave's first 1 KiB B request, per buffer
    int b_fill_off, b_read_off;        // NB > 2: byte offsets of the ring buffers being filled / read next (wave-uniform)
    // Byte offsets of this thread's global loads relative to the current K-step.  They never
    // change: the K-step advance is applied to the (scalar) buffer descriptors instead, base up and
    // size down, so the hardware range check keeps masking panels past the last of A and rows >= K of B, and no
    // vector register that a memory instruction has just read is written right after it.
    int a_moff[S::RHO][APTN], a_eoff[S::RHO][APTN], b_off[BPTN];
    // ADMA, ROLE 2: byte offsets of this lane's raw requests (mantissas: request e of sub-tile sub; exponents) in the
    // planes, relative to the K-step the A descriptors point at; LDS address of this wave's first mantissa request
    // and of its exponent request in raw buffer 0.  ROLE 1: where this thread reads its first chunk and its exponent
    // dword in raw buffer 0 (chunk i: 4 KiB / 512 bytes further on).
    int raw_moff[S::RHO][RQM], raw_eoff[S::RHO];
    char *raw_req_m, *raw_req_e;
    const char *raw_rd_m, *raw_rd_e;
    const int8_t *am_ptr;              // start of the K-step the next A fetch belongs to
    const uint8_t *ae_ptr;
    const uint16_t *b_ptr;             // start of the K-step the next B fetch belongs to
    int am_left, ae_left;              // bytes from those starts to the end of the planes
    int64_t b_left;                    // likewise for B, which may be larger than 2^31 bytes
    int e_shift;                       // bit position of this thread's exponent byte(s) in the loaded dword
    unsigned a_mask;                   // SK: bit sub * APT + i set if chunk i of sub-tile sub has a row < M in this wave
    // B in BFP16: this thread's chunks of the B^T tile (row n, 16 mantissas), like the A members
    char *bt_wr[2];
    const char *bt_rd[2];
    const char *bt_rdk[S::KS];         // ASWZ: fragment read address per k-slice, in B^T buffer 0, column block 0
    int bt_d1;                         // ASWZ: +16 or -16, where the second piece of this thread's chunk of the B^T tile sits (bt_wr points at the first)
    int bt_moff[BTPTN], bt_eoff[BTPTN];
    const int8_t *bm_ptr;
    const uint8_t *be_ptr;
    int bm_left, be_left, eb_shift;
    intx4 bt_mant[2][BTPTN];
    unsigned bt_expo[2][BTPTN];

    typedef float accv __attribute__((ext_vector_type(S::ACC)));
    accv acc[MTW][S::HB][S::NC];       // [band][row block of the band][column block]
    bf16x8 bfrag[S::KS][S::NC];        // this wave's slice of the resident B tile
    bf16x8 afrag[2][S::HB][S::KS];     // A fragments of the current and the next band: [band parity][row block][k-slice]
    intx4 a_mant[S::PF][APTN];
    unsigned a_expo[S::PF][APTN];
    intx4 b_raw[BPTN];
    unsigned dec[4];                   // bf16 pairs of the BFP16 block being decoded
    float cvf[2][2], ldf[2][2];        // decode pipeline: converted and scaled pairs in flight
    int shift;

    ATB_DEV TileKernel(const GemmParams &p_, char *lds, int t_first, int t_stride_) : p(p_), t_stride(t_stride_)
    {
        kt_steps = (p.K + S::T_K * S::KU - 1) / (S::T_K * S::KU) * S::KU;
        tid = threadIdx.x;
        lane = tid & 63;
        const int wave = tid >> 6;
        if constexpr (SKEWED) {      // wave row = wave group; wm only places the fragment reads and the stores, where the band carries the row
            wm = 0;
            wn = wave % S::WN;
        } else {
            wm = wave % S::WM;
            wn = wave / S::WM;
        }
        const int stid = tid % NTS;                  // index within the threads that share this staging job
        const int a_row = PAIRK ? stid / 2 : stid / A_CPR;
        const int a_q = PAIRK ? 2 * (stid % 2) : stid % A_CPR;           // first chunk of this thread in its row
        e_shift = ((((a_q * ACE) % kPanelK) / 8) & 3) * 8;
        // B staging.  The tile is row-major in LDS ([k][n], no padding), cut into slabs of NTS
        // 16-byte slots.  Request i of this wave group fills slab B_FIRST + i: wave w of the group
        // the 1 KiB at slot 64 w of the slab, lane l the slot l of that.  Chunk c of row k is stored at chunk position c ^ b_swz(k) of its row, so
        // that the rows a transposing read touches fall into different banks.
        const int slot0 = B_FIRST * NTS + __builtin_amdgcn_readfirstlane(wave % (NTS / 64)) * 64;
        const int blk = lane >> 4, j = lane & 15, r = j >> 2;
#pragma unroll
        for (int b = 0; b < S::AB; ++b) {
            char *a_base = lds + b * S::A_BYTES;
            if constexpr (S::ASWZ) {
                // piece c of row r sits at position c ^ (r % 8); a thread's rows are a multiple of 8 apart, so one swizzle
                // serves them all.  a_wr points at the first piece of the thread's run of 2 or 4; the others: a_d.
                const int row = a_row + A_FIRST * (NTS / A_CPR), swz = row & 7;
                a_wr[b] = a_base + row * S::PA + (((a_q * (ACE / 8)) ^ swz) * 16);
            } else {
                a_wr[b] = a_base + (a_row + A_FIRST * (NTS / A_CPR)) * S::PA + a_q * (ACE * 2);
            }
            // A fragment: lane l reads row l%MB of a row block, k = ks*KM + 8*(l/MB) .. +7
            a_rd[b] = a_base + (wm * 32 + lane % S::MB) * S::PA + (lane / S::MB) * 16;
        }
#pragma unroll
        for (int pc = 0; pc < 4; ++pc) a_d[pc] = pc * 16;
        bt_d1 = 16;
        if constexpr (S::ASWZ) {
            static_assert(!S::ASWZ || (ACE == 16 && (NTS / A_CPR) % 8 == 0), "swizzled A staging: chunks of two 16-byte pieces; a thread's rows share one swizzle");
            const int wrow = a_row + A_FIRST * (NTS / A_CPR);
            const int sx = ((wrow & 7) & ((PAIRK ? 4 : 2) - 1)) * 16;       // the swizzle's bits inside the run
#pragma unroll
            for (int pc = 0; pc < 4; ++pc) a_d[pc] = ((pc * 16) ^ sx) - sx;
            const int rrow = wm * 32 + lane % S::MB, rswz = rrow & 7;             // the same for a second row block, 16 rows on
#pragma unroll
            for (int ks = 0; ks < S::KS; ++ks) a_rdk[ks] = lds + rrow * S::PA + ((((S::KM / 8) * ks + lane / S::MB) ^ rswz) * 16);
        }
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            char *b_base = lds + S::AB * S::A_BYTES + b * B_BYTES;
            b_req[b] = b_base + slot0 * 16;
            b_wr[b] = b_req[b] + lane * 16;
            // B fragment through ds_read_b64_tr_b16: within each group of 16 lanes, lane i addresses
            // 4 consecutive columns of row i/4 (8 bytes, half a chunk), and lane j receives column j
            // of those 4 rows; a second read, 4 rows on, completes the lane's 8 k values.
            // MB = 32: groups 0, 1 of the wave's four groups of 16 lanes take the two halves of the 32 columns, rows
            // 0 .. 3 of the k-slice, groups 2, 3 the same columns of rows 8 .. 11.
            // MB = 16: group g takes the rows 8 g .. 8 g + 3 of the k-slice, all groups the same 16 columns.
            // The swizzle permutes the chunk index, so each of the first NBASE column blocks gets its own per-lane
            // base; block nt >= 4 (MB = 32 only) adds (nt / 4) * 256 bytes.
#pragma unroll
            for (int e = 0; e < NRD; ++e) {
                if constexpr (BTR) {
                    // B^T tile [n][k]: lane l reads column (row of B^T) wn*NC*MB + l%MB and the chunk of k-slice e
                    // (e = ks: 8 k values from KM ks + 8 (l/MB)); the chunk sits at position chunk ^ ((n / 2) % 8)
                    // of its row.  Sixteen lanes (rows n .. n+15) then cover all 64 banks once: row pairs differ in
                    // the position, the two rows of a pair in the half of the banks (pitch 128 bytes).
                    const int n = wn * S::NC * S::MB + lane % S::MB;
                    b_rd[b][e] = b_base + n * PBT + ((((S::KM / 8) * e + lane / S::MB) ^ ((n >> 1) & 7)) * 16);
                } else if constexpr (S::MB == 32) {
                    const int chunk = 4 * (wn * S::NC + e) + 2 * (blk & 1) + ((j & 3) >> 1), row = 8 * (blk >> 1) + r;
                    b_rd[b][e] = b_base + row * S::PB + ((chunk ^ S::b_swz(row)) * 16) + (j & 1) * 8;
                } else {
                    const int chunk = 2 * (wn * S::NC + e) + ((j & 3) >> 1), row = 8 * blk + r;
                    b_rd[b][e] = b_base + row * S::PB + ((chunk ^ S::b_swz(row)) * 16) + (j & 1) * 8;
                }
            }
        }
        if constexpr (BBFP) {
            // staging: thread -> (row n = stid / 4 + 64 i, chunk q = stid % 4 ... ) for T_K = 64; in general T_K / 16 chunks per row
            constexpr int CPR = S::T_K / 16;
            const int b_row = stid / CPR, b_q = stid % CPR;
            eb_shift = ((((b_q * 16) % kPanelK) / 8) & 3) * 8;
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                char *b_base = lds + S::AB * S::A_BYTES + b * B_BYTES;
                bt_wr[b] = b_base + b_row * S::PBF + (S::ASWZ ? ((2 * b_q) ^ (b_row & 7)) * 16 : b_q * 32);
                // B fragment: lane l reads column (row of B^T) l%MB of a column block, k = ks*KM + 8*(l/MB) .. +7
                bt_rd[b] = b_base + (wn * S::NC * S::MB + lane % S::MB) * S::PBF + (lane / S::MB) * 16;
            }
            if constexpr (S::ASWZ) {
                static_assert(!S::ASWZ || (NTS / CPR) % 8 == 0, "a thread's rows of the B^T tile share one swizzle");
                bt_d1 = (b_row & 1) ? -16 : 16;
                const int n = wn * S::NC * S::MB + lane % S::MB;
#pragma unroll
                for (int ks = 0; ks < S::KS; ++ks)
                    bt_rdk[ks] = lds + S::AB * S::A_BYTES + n * S::PBF + ((((S::KM / 8) * ks + lane / S::MB) ^ (n & 7)) * 16);
            }
            // rows >= N of B^T lie beyond the end of the planes and read as zero
#pragma unroll
            for (int i = 0; i < BTPT; ++i) {
                const int grow = b_row + i * (NTS / CPR);
                const int pnl = (b_q * 16) / kPanelK, kin = (b_q * 16) % kPanelK;
                bt_moff[i] = (pnl * p.N + grow) * kPanelK + kin;
                bt_eoff[i] = (pnl * p.N + grow) * (kPanelK / 8) + ((kin / 8) & ~3);
            }
        }
        // Offsets of sub-tile 0 / K-step 0 in the K-panel-major planes: the chunks of a sub-tile follow
        // each other in memory in the order of the staging threads, so a wave's request is one
        // contiguous KiB.  Rows >= M run into the next panel's rows (or past the end of the plane, which
        // reads as zero): they only feed rows of C that are never stored.  The tail of the last panel
        // (k >= K) is zero by the layout's contract, panels past the last read as zero.
#pragma unroll
        for (int sub = 0; sub < S::RHO; ++sub)
#pragma unroll
            for (int i = 0; i < APT; ++i) {
                const int grow = sub * S::T_MA + a_row + (PAIRK ? 0 : (A_FIRST + i) * (NTS / A_CPR));
                const int cq = PAIRK ? a_q + i : a_q;                  // chunk index within the row
                const int pnl = (cq * ACE) / kPanelK, kin = (cq * ACE) % kPanelK;
                a_moff[sub][i] = (pnl * p.M + grow) * kPanelK + kin;
                a_eoff[sub][i] = (pnl * p.M + grow) * (kPanelK / 8) + ((kin / 8) & ~3);
            }
        // B rows >= K lie beyond the end of B and read as zero; columns >= N wrap into the next row
        // and only feed output columns that are never stored.
#pragma unroll
        for (int i = 0; i < BPT; ++i) {
            const int slot = slot0 + i * NTS + lane;
            if constexpr (BTR) {
                // slot = 8 * (row n of the B^T tile) + chunk position: the chunk stored there is position ^ ((n / 2) % 8).
                // Offsets are relative to the tile's first row and the K-step's first k, both of which live in the
                // descriptor's base (open_b, load_b_chunk).  Rows >= N lie beyond the end of B^T and read as zero; k >= K
                // runs into the next row, whose (finite) values meet the zero tail of A.
                const int row = slot / (S::T_K / 8), c = (slot % (S::T_K / 8)) ^ ((row >> 1) & 7);
                b_off[i] = (row * p.K + c * 8) * 2;
            } else {
                const int row = slot / S::B_CPR, c = (slot % S::B_CPR) ^ S::b_swz(row);
                b_off[i] = (row * p.N + c * 8) * 2;
            }
        }
#pragma unroll
        for (int a = 0; a < MTW; ++a)
#pragma unroll
            for (int b = 0; b < S::HB * S::NC; ++b)
#pragma unroll
                for (int v = 0; v < S::ACC; ++v) acc[a][b / S::NC][b % S::NC][v] = 0.0f;
        if constexpr (ADMA_ON) {
            char *raw_base = lds + S::AB * S::A_BYTES + S::NB * S::B_BYTES;
            const int w = __builtin_amdgcn_readfirstlane(wave & 3);
            // a sub-tile's T_MA x 64 mantissa bytes are one contiguous run of the plane, cut into 1 KiB requests that
            // the four waves of the group take in turn; its T_MA x 8 exponent bytes are four requests of 256 bytes
            raw_req_m = raw_base + w * 1024;
            raw_req_e = raw_base + S::T_MA * kPanelK + w * 256;
#pragma unroll
            for (int sub = 0; sub < S::RHO; ++sub) {
#pragma unroll
                for (int e = 0; e < RQM; ++e) raw_moff[sub][e] = sub * S::T_MA * kPanelK + (e * 4 + w) * 1024 + lane * 16;
                raw_eoff[sub] = sub * S::T_MA * (kPanelK / 8) + w * 256 + lane * 4;
            }
            // chunk c = i * NTS + stid of the sub-tile is row c / 4, 16 mantissas from 16 (c % 4): byte 16 c of the raw
            // mantissas (consecutive lanes, consecutive 16 bytes); its two exponents sit in dword (c % 4) / 2 of the row's 8
            raw_rd_m = raw_base + stid * 16;
            raw_rd_e = raw_base + S::T_MA * kPanelK + (stid / 4) * (kPanelK / 8) + ((stid % 4) / 2) * 4;
        }
        // the offsets above are those of the tile at row 0, column 0; the streams move them to their tiles
        a_m0 = 0;
        b_n0 = 0;
        c_t = t_first;
        tile_at(c_t, m0, n0);
        if constexpr ((APT > 0 && !ADMA_ON) || RQ > 0) { open_a(t_first); remake_a(); }
        a_mask = 0xFFFFFFFFu;
        if constexpr (SK) {
            const int wrow = __builtin_amdgcn_readfirstlane(a_row);     // smallest staging row of this wave
            a_mask = 0;
#pragma unroll
            for (int sub = 0; sub < S::RHO; ++sub)
#pragma unroll
                for (int i = 0; i < APT; ++i) {
                    const int first = m0 + sub * S::T_MA + wrow + (PAIRK ? 0 : (A_FIRST + i) * (NTS / A_CPR));
                    if (first < p.M) a_mask |= 1u << (sub * APT + i);
                }
        }
        if constexpr (BTPT > 0) { open_b(t_first); remake_bt(); }
        if constexpr (BPT > 0) { open_b(t_first); remake_b(); }
    }

    ATB_DEV bool tile_at(int t, int &tm0, int &tn0) const { return tile_origin<S>(p, t, tm0, tn0); }

    // Point the A requests at the first K-step of tile t of the walk; past the last tile they get
    // empty buffers, so every request reads zeros without touching memory.  (The caller rebuilds
    // the descriptors.)
    ATB_DEV void open_a(int t)
    {
        int tm0 = 0, tn0 = 0;
        a_t = t;
        am_ptr = p.Am;
        ae_ptr = p.Ae;
        if (tile_at(t, tm0, tn0)) {
            const int d = tm0 - a_m0;
            a_m0 = tm0;
#pragma unroll
            for (int sub = 0; sub < S::RHO; ++sub)
#pragma unroll
                for (int i = 0; i < APT; ++i) {
                    a_moff[sub][i] += d * kPanelK;
                    a_eoff[sub][i] += d * (kPanelK / 8);
                }
            if constexpr (RQ > 0) {
#pragma unroll
                for (int sub = 0; sub < S::RHO; ++sub) {
#pragma unroll
                    for (int e = 0; e < RQM; ++e) raw_moff[sub][e] += d * kPanelK;
                    raw_eoff[sub] += d * (kPanelK / 8);
                }
            }
            am_left = p.k_panels * p.M * kPanelK;
            ae_left = p.k_panels * p.M * (kPanelK / 8);
            a_steps = kt_steps;
        } else {
            am_left = ae_left = 0;
            a_steps = 0x7fffffff;
        }
    }

    // The same for the B requests (bf16 B, or B^T in BFP16).
    ATB_DEV void open_b(int t)
    {
        int tm0 = 0, tn0 = 0;
        b_t = t;
        const bool live = tile_at(t, tm0, tn0);
        const int d = live ? tn0 - b_n0 : 0;
        b_n0 += d;
        b_steps = live ? kt_steps : 0x7fffffff;
        if constexpr (BBFP) {
            bm_ptr = p.Bm;
            be_ptr = p.Be;
            bm_left = live ? p.k_panels * p.N * kPanelK : 0;
            be_left = live ? p.k_panels * p.N * (kPanelK / 8) : 0;
#pragma unroll
            for (int i = 0; i < BTPT; ++i) {
                bt_moff[i] += d * kPanelK;
                bt_eoff[i] += d * (kPanelK / 8);
            }
        } else if constexpr (BTR) {
            // the tile's first row goes into the base, not into the offsets: rows are K elements apart, and 32-bit
            // offsets from the start of B^T would not reach the far end of a large operand
            b_ptr = p.B + (int64_t)(live ? tn0 : 0) * p.K;
            b_left = live ? ((int64_t)p.N - tn0) * p.K * 2 : 0;
        } else {
            b_ptr = p.B;
            b_left = live ? (int64_t)p.K * p.N * 2 : 0;
#pragma unroll
            for (int i = 0; i < BPT; ++i) b_off[i] += d * 2;
        }
    }

    // ---- global -> registers -------------------------------------------------------------
    // Descriptors are wave-uniform by construction; saying so keeps them in scalar registers.
    template <class T>
    ATB_DEV __amdgpu_buffer_rsrc_t make_rsrc(const T *ptr, int bytes)
    {
        const uint64_t a = reinterpret_cast<uint64_t>(ptr);
        const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)a);
        const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32));
        void *u = reinterpret_cast<void *>(((uint64_t)hi << 32) | lo);
        return __builtin_amdgcn_make_buffer_rsrc(u, 0, __builtin_amdgcn_readfirstlane(bytes), kRsrcFlags);
    }

    ATB_DEV void remake_a()
    {
        if constexpr (RQ > 0) {
            const uint64_t m = reinterpret_cast<uint64_t>(am_ptr), e = reinterpret_cast<uint64_t>(ae_ptr);
            rs.am_words = intx4{__builtin_amdgcn_readfirstlane((int)(uint32_t)m), __builtin_amdgcn_readfirstlane((int)(uint32_t)(m >> 32) & 0xFFFF),
                                __builtin_amdgcn_readfirstlane(am_left), kRsrcFlags};
            rs.ae_words = intx4{__builtin_amdgcn_readfirstlane((int)(uint32_t)e), __builtin_amdgcn_readfirstlane((int)(uint32_t)(e >> 32) & 0xFFFF),
                                __builtin_amdgcn_readfirstlane(ae_left), kRsrcFlags};
        } else {
            rs.am = make_rsrc(am_ptr, am_left);
            rs.ae = make_rsrc(ae_ptr, ae_left);
        }
    }

    // The A request stream moves on by one K-step (or to the workgroup's next tile) and rebuilds its descriptors.
    ATB_DEV void advance_a()
    {
        if (--a_steps == 0) {
            open_a(a_t + t_stride);
        } else {
            am_ptr += (S::T_K / kPanelK) * p.M * kPanelK;
            ae_ptr += (S::T_K / kPanelK) * p.M * (kPanelK / 8);
            am_left = max(am_left - (S::T_K / kPanelK) * p.M * kPanelK, 0);
            ae_left = max(ae_left - (S::T_K / kPanelK) * p.M * (kPanelK / 8), 0);
        }
        remake_a();
    }

    // ADMA, ROLE 2: request e of sub-tile `sub` of the K-step the A descriptors point at, straight into raw buffer
    // `slot` (e < RQM: 1 KiB of mantissas; e == RQM: this wave's 256 bytes of exponents).  Hand-issued like the B
    // requests (see load_b_chunk).  After the last request of the K-step's last sub-tile the descriptors move on.
    template <int slot, int sub, int e>
    ATB_DEV void load_raw_chunk()
    {
#if defined(__HIP_DEVICE_COMPILE__)
        int m0_saved;
        if constexpr (e < RQM) {
            const unsigned lds_addr = (unsigned)reinterpret_cast<uintptr_t>(raw_req_m + slot * S::RAW_BYTES + e * 4096);
            asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tbuffer_load_dwordx4 %2, %3, 0 offen lds\n\ts_mov_b32 m0, %0"
                         : "=&s"(m0_saved)
                         : "s"(__builtin_amdgcn_readfirstlane((int)lds_addr)), "v"(raw_moff[sub][e]), "s"(rs.am_words) : "memory");
        } else {
            const unsigned lds_addr = (unsigned)reinterpret_cast<uintptr_t>(raw_req_e + slot * S::RAW_BYTES);
            asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tbuffer_load_dword %2, %3, 0 offen lds\n\ts_mov_b32 m0, %0"
                         : "=&s"(m0_saved)
                         : "s"(__builtin_amdgcn_readfirstlane((int)lds_addr)), "v"(raw_eoff[sub]), "s"(rs.ae_words) : "memory");
        }
#endif
        if constexpr (sub == S::RHO - 1 && e == RQM) advance_a();
    }

    template <int x, int e = 0>
    ATB_DEV void load_raw()        // prologue: all requests of sub-tile x
    {
        if constexpr (e < RQ) {
            load_raw_chunk<x % S::NR, x % S::RHO, e>();
            load_raw<x, e + 1>();
        }
    }

    template <int x = 0>
    ATB_DEV void load_raw_first()
    {
        if constexpr (x < RAW_LEAD) {
            load_raw<x>();
            load_raw_first<x + 1>();
        }
    }

    // a K-step's offsets stay below 2^31, so a longer remainder may be cut off there
    ATB_DEV void remake_b()
    {
        const int bytes = (int)min(b_left, (int64_t)0x7fffffff);
        rs.b = make_rsrc(b_ptr, bytes);
        if constexpr (ASM_DMA) {
            const uint64_t a = reinterpret_cast<uint64_t>(b_ptr);
            rs.b_words = intx4{__builtin_amdgcn_readfirstlane((int)(uint32_t)a), __builtin_amdgcn_readfirstlane((int)(uint32_t)(a >> 32) & 0xFFFF),
                               __builtin_amdgcn_readfirstlane(bytes), kRsrcFlags};
        }
    }

    ATB_DEV void remake_bt()
    {
        rs.bm = make_rsrc(bm_ptr, bm_left);
        rs.be = make_rsrc(be_ptr, be_left);
    }

    // Chunk i of the BFP16 B tile the B descriptors point at, into register set `set`; after the
    // last chunk the descriptors move on to the next K-step.
    template <int set, int i>
    ATB_DEV void load_bt_chunk()
    {
        bt_mant[set][i] = __builtin_amdgcn_raw_buffer_load_b128(rs.bm, bt_moff[i], 0, 0);
        bt_expo[set][i] = __builtin_amdgcn_raw_buffer_load_b32(rs.be, bt_eoff[i], 0, 0);
        if constexpr (i == BTPT - 1) {
            if (--b_steps == 0) {
                open_b(b_t + t_stride);
            } else {
                bm_ptr += (S::T_K / kPanelK) * p.N * kPanelK;
                be_ptr += (S::T_K / kPanelK) * p.N * (kPanelK / 8);
                bm_left = max(bm_left - (S::T_K / kPanelK) * p.N * kPanelK, 0);
                be_left = max(be_left - (S::T_K / kPanelK) * p.N * (kPanelK / 8), 0);
            }
            remake_bt();
        }
    }

    template <int set, int i = 0>
    ATB_DEV void load_bt()
    {
        if constexpr (i < BTPT) {
            load_bt_chunk<set, i>();
            load_bt<set, i + 1>();
        }
    }

    // Chunk i of sub-tile `sub` of the K-step the A descriptors point at, into register set `set`.
    // After the last chunk of the last sub-tile the descriptors move on to the next K-step.
    // ADMA (ROLE 1): the chunk comes from raw buffer `slot` in LDS instead; the request stream is the other group's.
    template <int set, int sub, int i, int slot = 0>
    ATB_DEV void load_a_chunk()
    {
        if constexpr (ADMA_ON) {
            a_mant[set][i] = *reinterpret_cast<const intx4 *>(raw_rd_m + slot * S::RAW_BYTES + i * (NTS * 16));
            a_expo[set][i] = *reinterpret_cast<const unsigned *>(raw_rd_e + slot * S::RAW_BYTES + i * (NTS / 4) * (kPanelK / 8));
            return;
        }
        if constexpr (ACE == 16) {
            a_mant[set][i] = __builtin_amdgcn_raw_buffer_load_b128(rs.am, a_moff[sub][i], 0, 0);
        } else {
            intx2 t = __builtin_amdgcn_raw_buffer_load_b64(rs.am, a_moff[sub][i], 0, 0);
            a_mant[set][i] = intx4{t.x, t.y, 0, 0};
        }
        // the aligned dword that holds this chunk's exponent byte(s): sub-dword loads are far slower
        if constexpr (!PAIRK || i == 0)
            a_expo[set][i] = __builtin_amdgcn_raw_buffer_load_b32(rs.ae, a_eoff[sub][i], 0, 0);
        if constexpr (sub == S::RHO - 1 && i == APT - 1) advance_a();
    }

    template <int set, int sub, int i = 0>
    ATB_DEV void load_a()
    {
        if constexpr (i < APT) {
            load_a_chunk<set, sub, i, set % S::NR>();      // (prologue: sub-tile `set`, raw buffer `set`)
            load_a<set, sub, i + 1>();
        }
    }

    // Request i of the next B tile in fetch order, destined for LDS buffer `buf`.
    // VEC (even N: dword-aligned rows): one 16-byte load per lane straight into LDS (no registers, no ds_write);
    // completion is awaited with wait_b_landed() before the barrier that publishes the tile.
    // !VEC (odd N, rows of B only 2-byte aligned): aligned loads into registers plus a funnel shift;
    // store_b_chunk() writes them to LDS later.
    template <int i>
    ATB_DEV void load_b_chunk(int buf)
    {
        if constexpr (VEC) {
#if defined(__HIP_DEVICE_COMPILE__)
            typedef __attribute__((address_space(3))) void lds_void;
            char *dst = (S::NB > 2) ? b_req[0] + b_fill_off : b_req[buf];
            if constexpr (ASM_DMA) {
                // Issued by hand so that the compiler does not know of it: it cannot tell the buffer being
                // filled from the one being read and puts a vmcnt(0) in front of every transposing fragment
                // read that follows a request it knows of -- a full memory round trip inside the K-step when
                // requests and fragment reads share a phase, as they do at rho = 1 (measured: the symmetric
                // 128 x 256 tile 522 -> 992 TFLOP/s).  Completion is awaited by wait_vm() before the publishing
                // barrier, as for the built-in form.  Requests the compiler does not count make its own vmcnt
                // waits stricter, which is harmless only for waves that request nothing else: waves that also
                // fetch A would await the B tile before every decode (measured: helper waves 10 - 20 % slower),
                // so only wave groups without A requests take this path.
                const unsigned lds_addr = (unsigned)reinterpret_cast<uintptr_t>(dst + i * (NTS * 16));
                // M0 (the LDS base of the request) is put back afterwards: the compiler reserves it for its own uses
                // and is not told about this one
                int m0_saved;
                asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tbuffer_load_dwordx4 %2, %3, 0 offen lds\n\ts_mov_b32 m0, %0"
                             : "=&s"(m0_saved)
                             : "s"(__builtin_amdgcn_readfirstlane((int)lds_addr)), "v"(b_off[i]), "s"(rs.b_words) : "memory");
            } else {
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs.b, (lds_void *)(dst + i * (NTS * 16)), 16, b_off[i], 0, 0, 0);
            }
#else
            (void)buf;   // the host pass only parses this function
#endif
        } else {
            // odd N: a chunk starts at an odd bf16 of its row as often as not.  Fetch the 5 aligned
            // dwords that contain it and shift by half a dword where needed.
            const int al = b_off[i] & ~3, sh = (b_off[i] & 2) * 8;
            const intx4 lo = __builtin_amdgcn_raw_buffer_load_b128(rs.b, al, 0, 0);
            const int hi = __builtin_amdgcn_raw_buffer_load_b32(rs.b, al + 16, 0, 0);
            b_raw[i] = intx4{(int)__builtin_amdgcn_alignbit((unsigned)lo.y, (unsigned)lo.x, sh),
                             (int)__builtin_amdgcn_alignbit((unsigned)lo.z, (unsigned)lo.y, sh),
                             (int)__builtin_amdgcn_alignbit((unsigned)lo.w, (unsigned)lo.z, sh),
                             (int)__builtin_amdgcn_alignbit((unsigned)hi, (unsigned)lo.w, sh)};
        }
        if constexpr (i == BPT - 1) {
            if (--b_steps == 0) {
                open_b(b_t + t_stride);
            } else if constexpr (BTR) {
                b_ptr += S::T_K;
                b_left = max(b_left - (int64_t)S::T_K * 2, (int64_t)0);
            } else {
                b_ptr += S::T_K * p.N;
                b_left = max(b_left - (int64_t)S::T_K * p.N * 2, (int64_t)0);
            }
            remake_b();
        }
    }

    template <int i = 0>
    ATB_DEV void load_b(int buf)
    {
        if constexpr (i < BPT) {
            load_b_chunk<i>(buf);
            load_b<i + 1>(buf);
        }
    }

    // Workgroup barrier between microkernels.  It publishes this wave's LDS stores (lgkmcnt) but,
    // unlike __syncthreads(), does not wait for memory requests in flight: the A sub-tiles being
    // fetched into registers and the B tile being fetched straight into the other LDS buffer stay
    // in flight across it (the B tile is awaited explicitly where it has to be complete).
    ATB_DEV void switch_barrier()
    {
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    }

    // Block until this lane's memory requests, except the `younger` most recent ones, have
    // completed (s_waitcnt vmcnt; requests complete in order).
    template <int younger>
    ATB_DEV void wait_vm()
    {
        static_assert(younger >= 0 && younger < 64, "vmcnt is a 6-bit counter");
        __builtin_amdgcn_s_waitcnt((younger & 15) | (7 << 4) | (15 << 8) | ((younger >> 4) << 14));
    }

    // ---- registers -> LDS ----------------------------------------------------------------
    // BFP16 decode of mantissa pairs (exact: |m| <= 127 has 7 significant bits, bf16 keeps 8), as a
    // three-stage software pipeline over the pairs [first, first + count) of register set `set`:
    // step u converts pair u to fp32 (two v_cvt_f32_i32 with a byte select), scales pair u-1 by its
    // block's 2^(E-133) (two v_ldexp_f32) and packs pair u-2 to bf16 (one v_cvt_pk_bf16_f32); after
    // the 4th pair of a BFP16 block the block goes to LDS (bf16, [row][k], pitch PA).  The five
    // instructions of a step do not depend on each other: issued back to back as one dependent chain
    // per pair they cost 6.5 cycles each next to MFMAs, independent ones 4.  count + 2 steps drain it.
    // ISB selects the BFP16 B tile (chunks of 16 mantissas) instead of the A sub-tile.
    template <bool ISB, int set, int first, int count, int u>
    ATB_DEV void decode_step(char *dst_base)
    {
        constexpr int PPC = ISB ? 8 : ACE / 2;                       // pairs per chunk
        constexpr int ROWS = ISB ? NTS / (S::T_K / 16) : NTS / A_CPR; // LDS rows between a thread's chunks
        if constexpr (u >= 2 && u - 2 < count) {
            constexpr int j = first + u - 2, i = j / PPC, t = j % PPC;
            union { bf16x2 v; unsigned w; } pk;
            pk.v = bf16x2{(__bf16)ldf[(u - 2) % 2][0], (__bf16)ldf[(u - 2) % 2][1]};
            dec[t % 4] = pk.w;
            if constexpr (t % 4 == 3) {
                // piece of this thread's run of its row: with PAIRK the run holds both chunks, else each chunk has its own row
                constexpr int piece = (!ISB && PAIRK) ? 2 * i + t / 4 : t / 4;
                char *dst = dst_base + ((!ISB && PAIRK) ? 0 : i * ROWS * (ISB ? S::PBF : S::PA)) +
                            (!S::ASWZ ? piece * 16 : ISB ? piece * bt_d1 : a_d[piece]);
                *reinterpret_cast<intx4 *>(dst) = intx4{(int)dec[0], (int)dec[1], (int)dec[2], (int)dec[3]};
            }
        }
        if constexpr (u >= 1 && u - 1 < count) {
            constexpr int j = first + u - 1, i = j / PPC, t = j % PPC;
            if constexpr (t % 4 == 0 || u == 1) {
                const unsigned e = ISB ? bt_expo[set][i] : a_expo[set][PAIRK ? 0 : i];
                const int bit = ISB ? eb_shift + 8 * (t / 4) : PAIRK ? 16 * i + 8 * (t / 4) : e_shift + 8 * (t / 4);
                shift = (int)((e >> bit) & 0xFFu) - 133;
            }
            ldf[(u - 1) % 2][0] = ldexpf(cvf[(u - 1) % 2][0], shift);
            ldf[(u - 1) % 2][1] = ldexpf(cvf[(u - 1) % 2][1], shift);
        }
        if constexpr (u < count) {
            constexpr int j = first + u, i = j / PPC, t = j % PPC;
            const int w = ISB ? bt_mant[set][i][t / 2] : a_mant[set][i][t / 2];
            cvf[u % 2][0] = mant_to_float(w, (t % 2) * 2);
            cvf[u % 2][1] = mant_to_float(w, (t % 2) * 2 + 1);
        }
    }

    // The skinny-tile variant of the decode (SK): one BFP16 block (8 mantissas -> 16 bytes of bf16 in LDS)
    // per call, behind one wave-uniform test of its chunk's liveness bit.
    template <int set, int b>
    ATB_DEV void decode_block(char *dst_base, unsigned live)
    {
        constexpr int BPC = ACE / 8;                                 // blocks per chunk
        constexpr int i = b / BPC, q = b % BPC;
        if ((live >> i) & 1u) {
            const unsigned e = a_expo[set][PAIRK ? 0 : i];
            const int bit = PAIRK ? 16 * i + 8 * q : e_shift + 8 * q;
            const int sh = (int)((e >> bit) & 0xFFu) - 133;
            unsigned out[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int w = a_mant[set][i][2 * q + t / 2];
                union { bf16x2 v; unsigned w; } pk;
                pk.v = bf16x2{(__bf16)ldexpf(mant_to_float(w, (t % 2) * 2), sh), (__bf16)ldexpf(mant_to_float(w, (t % 2) * 2 + 1), sh)};
                out[t] = pk.w;
            }
            char *dst = dst_base + (PAIRK ? i * (ACE * 2) : i * (NTS / A_CPR) * S::PA) + q * 16;
            *reinterpret_cast<intx4 *>(dst) = intx4{(int)out[0], (int)out[1], (int)out[2], (int)out[3]};
        }
    }

    template <bool ISB, int set, int first, int count, int u = 0>
    ATB_DEV void decode_all(char *dst_base)
    {
        if constexpr (count > 0 && u < count + 2) {
            decode_step<ISB, set, first, count, u>(dst_base);
            decode_all<ISB, set, first, count, u + 1>(dst_base);
        }
    }

    template <int i>
    ATB_DEV void store_b_chunk(char *b_dst)
    {
        *reinterpret_cast<intx4 *>(b_dst + i * (NTS * 16)) = b_raw[i];
    }

    template <int set>
    ATB_DEV void store_a_all(char *a_dst) { decode_all<false, set, 0, NPAIR>(a_dst); }

    template <int set>
    ATB_DEV void store_bt_all(char *b_dst) { decode_all<true, set, 0, NPAIR_B>(b_dst); }

    template <int i = 0>
    ATB_DEV void store_b_all(char *b_dst)
    {
        if constexpr (i < BPT) {
            store_b_chunk<i>(b_dst);
            store_b_all<i + 1>(b_dst);
        }
    }

    // ---- LDS -> registers ----------------------------------------------------------------
    // B fragment (ks, nt) from LDS buffer `buf`: per lane l, column (wn*NC + nt)*MB + l%MB and
    // k = ks*KM + 8*(l/MB) .. +7.
    template <int ks, int nt>
    ATB_DEV void read_b_frag(int buf)
    {
        if constexpr (BBFP) {
            if constexpr (S::ASWZ)
                bfrag[ks][nt] = *reinterpret_cast<const bf16x8 *>(bt_rdk[ks] + buf * B_BYTES + nt * S::MB * S::PBF);
            else
                bfrag[ks][nt] = *reinterpret_cast<const bf16x8 *>(bt_rd[buf] + nt * S::MB * S::PBF + ks * S::KM * 2);
        } else if constexpr (BTR) {
            const char *base = (S::NB > 2) ? b_rd[0][ks] + b_read_off : b_rd[buf][ks];
            bfrag[ks][nt] = *reinterpret_cast<const bf16x8 *>(base + nt * S::MB * PBT);
        } else {
            const char *base = (S::NB > 2) ? b_rd[0][nt % S::NBASE] + b_read_off : b_rd[buf][nt % S::NBASE];
            const char *src = base + ks * S::KM * S::PB + (nt / S::NBASE) * (S::NBASE * 64);
            typedef __attribute__((address_space(3))) shortx4 lds_shortx4;
            union { shortx4 s[2]; bf16x8 b; } u;
            u.s[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_shortx4 *)(src));
            u.s[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_shortx4 *)(src + 4 * S::PB));
            bfrag[ks][nt] = u.b;
        }
    }

    template <int f = 0>
    ATB_DEV void read_b_frags_all(int buf)
    {
        if constexpr (f < S::KS * S::NC) {
            read_b_frag<f / S::NC, f % S::NC>(buf);
            read_b_frags_all<f + 1>(buf);
        }
    }

    // A fragment (band bd of the sub-tile as band(s, il) gives it, row block h of the band, k-slice ks).  In the
    // even deal the bands of the C tile go round-robin to the wave rows: this wave reads band il*WM + wm of the
    // sub-tile (wm is in a_rd).  The fragments of consecutive bands (counted across sub-tiles) alternate between
    // the two halves of afrag: `par` is that running band index mod 2.
    template <int par, int bd, int h, int ks>
    ATB_DEV void read_a_frag(int buf)
    {
        if constexpr (S::ASWZ)       // the k-slice's chunk position depends on the row: one address per k-slice, buffer and band as constants
            afrag[par][h][ks] = *reinterpret_cast<const bf16x8 *>(a_rdk[ks] + buf * S::A_BYTES + (bd * 32 + h * S::MB) * S::PA);
        else
            afrag[par][h][ks] = *reinterpret_cast<const bf16x8 *>(a_rd[buf] + (bd * 32 + h * S::MB) * S::PA + ks * S::KM * 2);
    }

    template <int par, int s, int f = 0>
    ATB_DEV void read_first_band(int buf)
    {
        if constexpr (f < S::HB * S::KS) {
            read_a_frag<par, band(s, 0), S::KIN ? f / S::KS : f % S::HB, S::KIN ? f % S::KS : f / S::HB>(buf);    // in the order of their first use
            read_first_band<par, s, f + 1>(buf);
        }
    }

    // ---- one microkernel, software-pipelined by hand ---------------------------------------
    // Side work of phase (kpar, s), in issue order: the memory requests for A sub-tile g+PF (and, in
    // the first phase of a K-step, for the B tile two K-steps ahead), the decode + LDS write of A
    // sub-tile g+1, and (last phase of the K-step) the LDS writes of the B tile fetched in the first.
    template <int s>
    static constexpr int n_side()
    {
        return RQ + APT + (s == 0 ? BPT + BTPT : 0) + NSTEP_A + NSTEP_B + ((!VEC && s + 1 == S::RHO) ? BPT : 0);
    }

    template <int ki, int s, int j>
    ATB_DEV void side()
    {
        constexpr int kpar = ki & 1;             // parity of the K-step: B buffers and B register sets
        constexpr int g = ki * S::RHO + s;       // running sub-tile index within the loop body
        constexpr int n_la = APT, n_lb = (s == 0 ? BPT : 0), n_lt = (s == 0 ? BTPT : 0), n_dt = NPAIR_B / S::RHO;
        // (the raw A requests come first: they are awaited a phase later, the B tile's only three phases later, and
        // requests complete in order)
        constexpr int j0 = RQ, j1 = j0 + n_lb, j2 = j1 + n_lt, j3 = j2 + n_la, j4 = j3 + NSTEP_A, j5 = j4 + NSTEP_B;
        if constexpr (j < j0) {
            load_raw_chunk<(g + RAW_LEAD) % S::NR, (s + RAW_LEAD) % S::RHO, j>();
        } else if constexpr (j < j1) {
            load_b_chunk<j - j0>(kpar);
        } else if constexpr (j < j2) {
            load_bt_chunk<kpar ^ 1, j - j1>();
        } else if constexpr (j < j3) {
            load_a_chunk<g % S::PF, (s + S::PF) % S::RHO, j - j2, (g + S::PF) % S::NR>();
        } else if constexpr (j < j4) {
            if constexpr (SK)
                decode_block<(g + S::DA) % S::PF, j - j3>(a_wr[(g + S::DA) % S::AB], a_mask >> (((s + S::DA) % S::RHO) * APTN));
            else
                decode_step<false, (g + S::DA) % S::PF, 0, NPAIR, j - j3>(a_wr[(g + S::DA) % S::AB]);
        } else if constexpr (j < j5) {
            decode_step<true, kpar, s * n_dt, n_dt, j - j4>(bt_wr[kpar]);
        } else {
            store_b_chunk<j - j5>((S::NB > 2) ? b_wr[0] + b_fill_off : b_wr[kpar]);
        }
    }

    template <int ki, int s, int j, int jend>
    ATB_DEV void side_range()
    {
        if constexpr (j < jend) {
            side<ki, s, j>();
            side_range<ki, s, j + 1, jend>();
        }
    }

    // Slot m: MG MFMAs back to back, then the slot's share of the side work; after the last column block of a
    // (k-slice, row block) the same A fragment of the next band; in the last band of the K-step a B fragment is
    // replaced by the next K-step's after its last use (second row block).  MFMAs that follow each other share their
    // A fragment or (Shape::KIN) their accumulator block.  The fences pin this order, so that the VALU decode and the
    // LDS traffic issue in the shadow of the MFMAs.
    static constexpr int MG = ATB_MFMA_GROUP;
    static_assert(S::NC % MG == 0 && (!S::KIN || S::KS % MG == 0), "a slot's MFMAs share one A fragment or one accumulator block");

    template <int ki, int s, int mm>
    ATB_DEV void slot_mfma()
    {
        constexpr int il = mm / (S::HB * S::KS * S::NC), ks = S::KIN ? mm % S::KS : (mm / (S::HB * S::NC)) % S::KS,
                      h = S::KIN ? (mm / (S::KS * S::NC)) % S::HB : (mm / S::NC) % S::HB, nt = S::KIN ? (mm / S::KS) % S::NC : mm % S::NC;
        constexpr int local = first_local(s) + il;            // accumulator band of this wave
        constexpr int par = (bands_before(ki * S::RHO + s) + il) % 2;       // which half of afrag this band uses
        if constexpr (S::MB == 16)
            acc[local][h][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bfrag[ks][nt], afrag[par][h][ks], acc[local][h][nt], 0, 0, 0);
        else
            acc[local][h][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfrag[ks][nt], afrag[par][h][ks], acc[local][h][nt], 0, 0, 0);
    }

    template <int ki, int s, int mm>
    ATB_DEV void slot_reads()
    {
        constexpr int il = mm / (S::HB * S::KS * S::NC), ks = S::KIN ? mm % S::KS : (mm / (S::HB * S::NC)) % S::KS,
                      h = S::KIN ? (mm / (S::KS * S::NC)) % S::HB : (mm / S::NC) % S::HB, nt = S::KIN ? (mm / S::KS) % S::NC : mm % S::NC;
        constexpr int g = ki * S::RHO + s;
        constexpr int par = (bands_before(g) + il) % 2;
        if constexpr (nt == S::NC - 1) {
            if constexpr (il + 1 < per(s))
                read_a_frag<par ^ 1, band(s, il + 1), h, ks>(g % S::AB);
            else if constexpr (S::AB == 4)      // first band of the next sub-tile, already complete in LDS
                read_a_frag<par ^ 1, band((s + 1) % S::RHO, 0), h, ks>((g + 1) % S::AB);
        }
        if constexpr (s + 1 == S::RHO && il + 1 == per(s) && h == S::HB - 1) read_b_frag<ks, nt>((ki & 1) ^ 1);
    }

    template <int ki, int s, int m>
    ATB_DEV void slots()
    {
        constexpr int nslot = nm(s) / MG;
        if constexpr (m < nslot) {
            constexpr int nside = n_side<s>();
            if constexpr (COMPUTE) {
                slot_mfma<ki, s, m * MG>();
                if constexpr (MG >= 2) slot_mfma<ki, s, m * MG + 1>();
                if constexpr (MG >= 4) { slot_mfma<ki, s, m * MG + 2>(); slot_mfma<ki, s, m * MG + 3>(); }
            }
            ATB_FENCE();
            // the last eighth of the slots carries no side work, so that the LDS stores of the decode
            // have drained when the wave reaches the switch barrier
            constexpr int NS = nslot - nslot / 8;
            constexpr int j0 = (m * nside) / NS < nside ? (m * nside) / NS : nside;
            constexpr int j1 = ((m + 1) * nside) / NS < nside ? ((m + 1) * nside) / NS : nside;
            side_range<ki, s, j0, j1>();
            if constexpr (COMPUTE) {
                slot_reads<ki, s, m * MG>();
                if constexpr (MG >= 2) slot_reads<ki, s, m * MG + 1>();
                if constexpr (MG >= 4) { slot_reads<ki, s, m * MG + 2>(); slot_reads<ki, s, m * MG + 3>(); }
            }
            ATB_FENCE();
            slots<ki, s, m + 1>();
        }
    }

    // Phase s of K-step ki of the loop body.
    template <int ki, int s>
    ATB_DEV void phases()
    {
        if constexpr (s < S::RHO) {
            constexpr int g = ki * S::RHO + s;
            if constexpr (S::AB == 2 && COMPUTE) read_first_band<bands_before(g) % 2, s>(g % 2);
            ATB_FENCE();
            slots<ki, s, 0>();
            // The B tile requested (straight into LDS) in the first phase of a K-step is read in the
            // last band of the next K-step, so the last barrier before that band has to publish it.
            // With NB buffers the tile read in K-step kt + 1 was requested at the start of K-step kt + 2 - NB.
            // rho = 1: the barrier is the one ending K-step kt; younger than the tile's requests are the A
            // requests of NB - 1 K-steps and NB - 2 further B tiles.  rho >= 2: the barrier ending the
            // last-but-one phase of K-step kt + 1; younger are the A requests of NB rho - 1 phases and
            // NB - 1 further B tiles.  (A smaller count only waits for more than necessary.)
            if constexpr (VEC && BPT > 0 && S::RHO == 1) wait_vm<vm_cap((S::NB - 1) * A_VMEM + (S::NB - 2) * BPT)>();
            // ADMA: the raw sub-tile requested in the previous phase is read by the other group in the next one, so
            // everything older than this phase's own requests has to have landed (which covers the B tile as well)
            if constexpr (RQ > 0) wait_vm<vm_cap(RQ + BPT)>();
            else if constexpr (VEC && BPT > 0 && S::RHO >= 2 && s == S::RHO - 2)
                wait_vm<vm_cap((S::NB * S::RHO - 1) * A_VMEM + (S::NB - 1) * BPT)>();
            switch_barrier();   // the "kernel switch" of the ATB nest
            phases<ki, s + 1>();
        }
    }

    static constexpr int vm_cap(int n) { return n < 63 ? n : 63; }     // vmcnt is a 6-bit counter

    // NB > 2: the ring moves on by one buffer per K-step
    ATB_DEV void advance_b_ring()
    {
        b_fill_off = (b_fill_off + B_BYTES == S::NB * B_BYTES) ? 0 : b_fill_off + B_BYTES;
        b_read_off = (b_read_off + B_BYTES == S::NB * B_BYTES) ? 0 : b_read_off + B_BYTES;
    }

    template <int ki>
    ATB_DEV void ksteps()
    {
        if constexpr (ki < S::KU) {
            phases<ki, 0>();
            if constexpr (S::NB > 2) advance_b_ring();
            ksteps<ki + 1>();
        }
    }

    template <int g = 0>
    ATB_DEV void prologue_loads()
    {
        if constexpr (g < S::PF) {
            load_a<g, g % S::RHO>();
            prologue_loads<g + 1>();
        }
    }

    ATB_DEV void run()
    {
        // prologue: the first NB B tiles into LDS, the first PF A sub-tiles into registers, sub-tile 0
        // into LDS, B tile 0 into fragment registers
        if constexpr (S::NB > 2) b_fill_off = 0;
        if constexpr (ADMA_ON) {
            // the first RAW_LEAD raw sub-tiles into the ring, landed and published before the decoding group reads them
            if constexpr (RQ > 0) load_raw_first();
            wait_vm<0>();
            __syncthreads();
        }
        load_b(0);
        if constexpr (BBFP) { load_bt<0>(); load_bt<1>(); }
        prologue_loads();
        if constexpr (!VEC) store_b_all(b_wr[0]);
        if constexpr (S::NB > 2) {
#pragma unroll
            for (int t = 1; t < S::NB; ++t) {
                b_fill_off = t * B_BYTES;
                load_b(0);
                if constexpr (!VEC) store_b_all(b_wr[0] + b_fill_off);
            }
        } else {
            load_b(1);
        }
        if constexpr (BBFP) {
            // B tiles 0 and 1 decoded into LDS; tile 2 into the register set that K-step 0 decodes
            store_bt_all<0>(bt_wr[0]);
            store_bt_all<1>(bt_wr[1]);
            load_bt<0>();
        }
        store_a_all<0>(a_wr[0]);
        if constexpr (S::AB == 4) store_a_all<1>(a_wr[1]);
        if constexpr (VEC && BPT > 0) wait_vm<0>();
        if constexpr (!VEC && S::NB == 2) store_b_all(b_wr[1]);
        __syncthreads();
        if constexpr (S::NB > 2) b_read_off = 0;
        if constexpr (COMPUTE) read_b_frags_all(0);
        if constexpr (S::NB > 2) {
            // K-step 0 refills buffer 0 and reads the fragments of K-step 1 from buffer 1
            b_fill_off = 0;
            b_read_off = B_BYTES;
        }
        // B buffer 0 is refilled from the first phase on: every wave must have its fragments first
        switch_barrier();
        if constexpr (S::AB == 4 && COMPUTE) read_first_band<0, 0>(0);

        // The number of K-steps is rounded up to a whole loop body: the extra steps multiply by B rows
        // >= K, which read as zero.  The last K-steps of a tile already request, decode and stage the
        // first operands of the workgroup's next tile (the request streams have moved on to it), so the
        // next tile needs no prologue: the epilogue is all that separates two tiles' arithmetic.
        for (;;) {
            for (int kt = 0; kt < kt_steps; kt += S::KU) ksteps<0>();
            if constexpr (!COMPUTE) { } else if constexpr (CBFP) store_c_bfp(); else store_c();
            c_t += t_stride;
            if (!tile_at(c_t, m0, n0)) break;
#pragma unroll
            for (int a = 0; a < MTW; ++a)
#pragma unroll
                for (int b = 0; b < S::HB * S::NC; ++b)
#pragma unroll
                    for (int v = 0; v < S::ACC; ++v) acc[a][b / S::NC][b % S::NC][v] = 0.0f;
        }
        // the requests past the end of the walk (they read zeros) target registers and LDS of this wave
        wait_vm<0>();
    }

    // 32-row band of the C tile that accumulator band a of this wave holds (without the wave row's offset wm of the even deal)
    static constexpr int band_of_acc(int a)
    {
        int s = 0;
        while (s + 1 < S::RHO && first_local(s + 1) <= a) ++s;
        return s * S::SMT + band(s, a - first_local(s));
    }

    // epilogue: fp32 -> bf16 (round to nearest even) and store, once per tile.  Lane l of block
    // (a, h, b) holds row l%MB of the block and, in registers 4g .. 4g+3, its columns 8g + 4*(l/MB) + 0..3
    // (MB = 32: g = 0..3; MB = 16: g = 0 only).
    ATB_DEV void store_c()
    {
        const bool st_vec = (p.N % 4) == 0;
#pragma unroll
        for (int a = 0; a < S::HB * MTW; ++a) {
            const int m = m0 + (band_of_acc(a / S::HB) + wm) * 32 + (a % S::HB) * S::MB + lane % S::MB;
#pragma unroll
            for (int b = 0; b < S::NC; ++b) {
                const int nb = n0 + (wn * S::NC + b) * S::MB + 4 * (lane / S::MB);
#pragma unroll
                for (int g = 0; g < S::ACC / 4; ++g) {
                    const int n = nb + 8 * g;
                    bf16x4 o;
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = (__bf16)acc[a / S::HB][a % S::HB][b][4 * g + e];
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

    // Epilogue for C in BFP16 (blocks of 8 along N): a block is the 4 consecutive columns of lane l
    // plus the 4 of lane l ^ MB (same row).  Same arithmetic as the stand-alone quantiser: shared
    // exponent = largest fp32 exponent field, mantissa = clamp(rne(x * 2^(133 - E)), +-127).
    // Needs N % 8 == 0; columns N .. 64 * n_panels - 1 (the tail of C's last panel) are written as zero.
    ATB_DEV void store_c_bfp()
    {
#pragma unroll
        for (int a = 0; a < S::HB * MTW; ++a) {
            const int m = m0 + (band_of_acc(a / S::HB) + wm) * 32 + (a % S::HB) * S::MB + lane % S::MB;
#pragma unroll
            for (int b = 0; b < S::NC; ++b) {
                const int nb = n0 + (wn * S::NC + b) * S::MB + 4 * (lane / S::MB);
#pragma unroll
                for (int g = 0; g < S::ACC / 4; ++g) {
                    const int n = nb + 8 * g;
                    const bool live = (n < p.N);           // whole blocks: N % 8 == 0
                    float x[4];
                    unsigned e = 0;
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        x[t] = live ? acc[a / S::HB][a % S::HB][b][4 * g + t] : 0.0f;
                        e = max(e, (__float_as_uint(x[t]) >> 23) & 0xFFu);
                    }
                    const unsigned other = (unsigned)__builtin_amdgcn_ds_bpermute((lane ^ S::MB) << 2, (int)e);
                    e = max(e, other);
                    const int sh = 133 - (int)e;
                    unsigned w = 0;
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        float r = rintf(ldexpf(x[t], sh));
                        r = fminf(fmaxf(r, -127.0f), 127.0f);
                        w |= ((unsigned)((int)r) & 0xFFu) << (8 * t);
                    }
                    if (m < p.M && n < p.n_panels * kPanelK) {
                        const int64_t rec = (int64_t)(n / kPanelK) * p.M + m;       // (panel, row)
                        *reinterpret_cast<unsigned *>(p.Cm + rec * kPanelK + n % kPanelK) = w;
                        if (((lane / S::MB) & 1) == 0) p.Ce[rec * (kPanelK / 8) + ((n % kPanelK) >> 3)] = (uint8_t)e;
                    }
                }
            }
        }
    }
};

// Workgroup -> C tiles (TileKernel::tile_at has the mapping).  For the large tiles the grid is
// persistent: it holds only as many workgroups as fit on the chip at once, and workgroup b serves
// tiles b / 8, b / 8 + gridDim.x / 8, ... of its XCD's run as one pipeline, so no tile waits for a
// workgroup launch or for its first operands.
template <class S, bool VEC, int ROLE, bool BBFP, bool CBFP, bool BTR>
__device__ __forceinline__ void tile_loop(const GemmParams &p, char *lds)
{
    const int total = p.tiles_m * p.tiles_n;
    const int per_xcd = (total + 7) / 8;
    const int first = (int)blockIdx.x / 8;
    if (first >= per_xcd || (int)(blockIdx.x % 8) * per_xcd + first >= total) return;   // the whole workgroup leaves
    // workgroups of the skinny-problem instances whose tile lies at least half beyond M take the variant
    // that skips dead rows (measured on the other small instances it does not pay: there a wave's chunks
    // are either all live or the block-wise decode costs more than the skipped rows save)
    if constexpr (S::T_K >= 256 && S::T_MC * S::T_N < 256 * 256 && !BBFP && !BTR) {
        int m0 = 0, n0 = 0;
        tile_origin<S>(p, first, m0, n0);
        if (p.M - m0 <= S::T_MC / 2) {
            TileKernel<S, VEC, ROLE, BBFP, CBFP, true> tile(p, lds, first, (int)gridDim.x / 8);
            tile.run();
            return;
        }
    }
    TileKernel<S, VEC, ROLE, BBFP, CBFP, false, BTR> tile(p, lds, first, (int)gridDim.x / 8);
    tile.run();
}

template <class S, bool VEC, bool BBFP = false, bool CBFP = false, bool BTR = false>
__global__ void __launch_bounds__(S::NT, S::OCC) atb_gemm_kernel(const GemmParams p)
{
    __shared__ __attribute__((aligned(16))) char lds[BBFP ? S::LDS_BYTES_BT : S::LDS_BYTES];
    if constexpr (S::HW > 0) {
        if (threadIdx.x < S::CW * 64)
            tile_loop<S, VEC, 4, BBFP, CBFP, BTR>(p, lds);
        else
            tile_loop<S, VEC, 3, BBFP, CBFP, BTR>(p, lds);
    } else if constexpr (S::CW == 8) {
        // wave-uniform branch; both sides execute the same sequence of barriers
        if (threadIdx.x < 256)
            tile_loop<S, VEC, 1, BBFP, CBFP, BTR>(p, lds);
        else
            tile_loop<S, VEC, 2, BBFP, CBFP, BTR>(p, lds);
    } else {
        tile_loop<S, VEC, 0, BBFP, CBFP, BTR>(p, lds);
    }
}

// Compute units of the current device (0 if there is none).  Looked up once per device; the table is
// guarded, so concurrent first launches from several threads are fine, and the lookup enqueues nothing
// (a first launch inside a stream capture is as good as any other).
inline int compute_units()
{
    constexpr int kMaxDevices = 64;
    static std::mutex guard;
    static int cached[kMaxDevices] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 0;
    std::lock_guard<std::mutex> lock(guard);
    if (cached[dev] == 0) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 8) return 0;
        cached[dev] = cus;
    }
    return cached[dev];
}

template <class S, bool VEC, bool BBFP, bool CBFP, bool BTR = false>
hipError_t launch_kernel(const GemmParams &p, hipStream_t stream)
{
    const int total = p.tiles_m * p.tiles_n;
    const int per_xcd = (total + 7) / 8;
    // Small tiles keep one workgroup per tile: several of them share a CU and overlap each other's
    // prologue and epilogue already, and the hardware dispatcher balances them better than a fixed walk.
    // The 256 x 256 tiles get a persistent grid of one workgroup per CU (the accumulators of one tile are half the
    // CU's 512 KiB of vector registers, so a second workgroup never fits beside the first, whatever the LDS
    // footprint): a grid larger than what is resident would only queue, a smaller one idles CUs.
    constexpr bool persistent = S::T_MC * S::T_N >= 256 * 256;
    static_assert(!persistent || 2 * (S::T_MC * S::T_N * 4) >= 512 * 1024, "the persistent grid assumes one workgroup per CU");
    int slots = per_xcd;                                                           // workgroups per XCD
    if (persistent) {
        const int cus = compute_units();
        if (cus == 0) return hipErrorNoDevice;
        slots = std::min(per_xcd, cus / 8);
    }
    hipLaunchKernelGGL((atb_gemm_kernel<S, VEC, BBFP, CBFP, BTR>), dim3(slots * 8), dim3(S::NT), 0, stream, p);
    return hipGetLastError();
}

template <class S>
hipError_t launch_instance(const GemmParams &p, hipStream_t stream)
{
    // 16-byte requests need dword-aligned addresses: B rows start at multiples of 2 N bytes, chunks at
    // multiples of 16 bytes within a row, so any even N qualifies (a chunk that straddles the end of
    // a row only feeds output columns >= N, which are never stored)
    if ((p.N % 2) == 0) return launch_kernel<S, true, false, false>(p, stream);
    return launch_kernel<S, false, false, false>(p, stream);
}

// The other storage formats (B and/or C in BFP16); C in BFP16 needs N % 8 == 0 (checked by the caller).
template <class S>
hipError_t launch_instance_fmt(const GemmParams &p, int b_format, int c_format, hipStream_t stream)
{
    const bool bb = (b_format == ATB_FMT_BFP16), cb = (c_format == ATB_FMT_BFP16);
    if (b_format == ATB_FMT_BF16_T) {
        // bf16 B handed over transposed: compiled for the tiles with K-steps of 64 and a bf16 C
        if constexpr (S::T_K == 64 && S::T_MC * S::T_N >= 128 * 256) {
            if (!cb) return launch_kernel<S, true, false, false, true>(p, stream);
        }
        return hipErrorInvalidValue;
    }
    if (bb && cb) return launch_kernel<S, true, true, true>(p, stream);
    if (bb) return launch_kernel<S, true, true, false>(p, stream);
    if (cb) return launch_kernel<S, true, false, true>(p, stream);
    return launch_kernel<S, true, false, false>(p, stream);
}

template <class S, bool FMT = false>
Instance make_instance(double eff_scale = 0.0, double lone_cap = 0.0)
{
    Instance i;
    i.eff_scale = eff_scale;
    i.lone_cap = lone_cap;
    i.T_MA = S::T_MA;
    i.T_MC = S::T_MC;
    i.T_K = S::T_K;
    i.T_N = S::T_N;
    i.wave_m = S::WM;
    i.wave_n = S::WN;
    i.threads = S::NT;
    i.lds_bytes = S::LDS_BYTES;
    // workgroups that share a CU: one for the 8-wave workgroups (two waves per SIMD that use more than a quarter of
    // the SIMD's registers each); for the others what the LDS footprint and the 8 wave slots of a SIMD admit
    i.wg_per_cu = (S::CW == 8) ? 1 : std::max(1, std::min(std::min(8, (160 * 1024) / S::LDS_BYTES), 8 * 256 / S::NT));
    if (S::OCC > 1) i.wg_per_cu = std::min(i.wg_per_cu, S::OCC * 256 / S::NT);      // compiled for OCC waves per SIMD: no more fit by registers
    i.mfma_rows = S::MB;
    i.launch = &launch_instance<S>;
    if constexpr (FMT) i.launch_fmt = &launch_instance_fmt<S>; else i.launch_fmt = nullptr;
    i.has_b_transposed = FMT && S::T_K == 64 && S::T_MC * S::T_N >= 128 * 256;
    return i;
}

// The instance table is cut into three groups so that the build can compile them side by side (one
// translation unit per group, -DATB_GROUP=0/1/2); without the macro this file holds all of them.
#ifndef ATB_GROUP
#define ATB_GROUP -1
#endif
#define ATB_IN_GROUP(g) (ATB_GROUP == -1 || ATB_GROUP == (g))

#ifndef ATB_ATB_B_RING
#define ATB_ATB_B_RING 2
#endif
// The symmetric 256 x 256 tile can have a third B buffer too, now that its A rows are not padded (64 + 96 KiB =
// exactly the CU's 160 KiB); a B tile then has two K-steps to arrive instead of one.  Measured on 8192^3 with the
// 32 x 32 x 16 MFMAs: -0.9 % (1260 against 1271 TFLOP/s, interleaved timing); the waves that await the B tile are
// not the ones the K-step waits for.  Build option -DATB_SYM_B_RING=3; the library ships with 2.
#ifndef ATB_SYM_B_RING
#define ATB_SYM_B_RING 2
#endif
#ifndef ATB_ATB_A_RING
#define ATB_ATB_A_RING 2
#endif
// Bands of the 256-row C tile that move from the decoding wave group to the other one (Shape::SKEW).
#ifndef ATB_SYM_SKEW
#define ATB_SYM_SKEW 0
#endif
#ifndef ATB_ATB_SKEW
#define ATB_ATB_SKEW 0
#endif
// A third use of the LDS that ATB frees at the 256 x 256 tile: a ring of four raw A sub-tiles (36 KiB at rho = 2)
// that the second wave group fills with requests straight into LDS, as it does for B, so that the decoding waves
// read their chunks from LDS instead of loading them from memory into registers (Shape::ADMA).  Parity-green and
// bit-equal; measured on 8192^3: -0.5 % (1261 against 1268 TFLOP/s, interleaved timing, the same clock): what the A
// loads cost is the bytes that come into the CU, whichever way they take.  Build option -DATB_ATB_RAW_RING=1.
#ifndef ATB_ATB_RAW_RING
#define ATB_ATB_RAW_RING 0
#endif

const Instance g_instances[] = {
#if ATB_IN_GROUP(0)
    // T_MC = T_N = 256, T_K = 64: the sweep over rho = 1, 2, 4, 8.
    // 8 waves (2 x 4, two per SIMD, 128 accumulator registers each) let one wave's decode and memory
    // instructions issue while the other's MFMAs run; T_MA = 32 only feeds a 1 x 4 grid.
    // Staging split (last two arguments): the first wave group decodes all of A and the second requests
    // all of B, by hand (see load_b_chunk) at rho <= 2.  (While the symmetric tile's B requests were the
    // built-in ones, a quarter of its A tile went to the second group: 1195 TFLOP/s against 950 for this
    // 4 : 0 split; with hand-issued requests 4 : 0 measures 1294 against 1243 for 3 : 1, on 8192^3.)
    // The A fetch runs one to one and a half K-steps ahead of its use at every rho (PF phases).
    // These three, and the mid-size and small tiles below, also come with B and/or C stored as BFP16
    // (the all-BFP16 configurations of Sec. 6.1); the 4-wave 256-row instances have no registers left for it.
    make_instance<Shape<256, 256, 64, 256, 2, 4, 2, 2, 4, 0, 2, ATB_SYM_B_RING, 0, ATB_SYM_SKEW>, true>(1.0),
    // What ATB's smaller A buffers free in LDS (36 KiB at rho = 2, 54 KiB at rho = 4) could hold a third B buffer
    // (ATB_ATB_B_RING = 3: 132 / 114 KiB; the symmetric tile cannot have one, 72 + 96 KiB) or a ring of four A
    // buffers whose decode runs two sub-tiles ahead, so that a microkernel's first fragments are read before the
    // switch barrier (ATB_ATB_A_RING = 4).  Measured on 8192^3, neither pays on this chip (B ring: -0.2 % / -0.9 %,
    // A ring: -3.8 % / -1.6 % at rho = 2 / 4): B tiles already arrive two K-steps after their request, and the
    // deeper A ring costs registers.  Both stay build options (-DATB_ATB_B_RING=3, -DATB_ATB_A_RING=4) for that
    // measurement; the library ships with 2 and 2.
    make_instance<Shape<128, 256, 64, 256, 2, 4, (ATB_ATB_A_RING == 4 ? 4 : 2), ATB_ATB_A_RING, 2, 0, 2, ATB_ATB_B_RING, 0, ATB_ATB_SKEW, 0, 1, (ATB_ATB_RAW_RING != 0 && ATB_ATB_A_RING == 2)>, true>(1.0),
    make_instance<Shape<64, 256, 64, 256, 2, 4, 4, ATB_ATB_A_RING, 1, 0, 2, ATB_ATB_B_RING>, true>(1.0),
    make_instance<Shape<32, 256, 64, 256, 1, 4, 8, 4>>(1.0),
    // T_K = 128 exists only with ATB: at rho = 8 the A buffers take 17 KiB next to 128 KiB of B; the
    // symmetric tile would need 264 KiB of LDS (the "ATB makes an infeasible tile legal" case of Sec. 6.3)
    make_instance<Shape<32, 256, 128, 256, 1, 4, 8, 2>>(),
#endif
#if ATB_IN_GROUP(1)
    // Mid-size tiles for problems with too few 256 x 256 tiles to fill 256 CUs (e.g. the N = 2048 shapes of the
    // paper's Table 3).  Their full-load throughput relative to the 256 x 256 family's fit comes from the
    // microkernel issue model where an instance has no first argument (the selector computes it: 0.84 for the
    // T_K = 128 instance above, 1.05 for the symmetric 128 x 128 tile; measured on 8192^3: 0.88, 1.08).
    // 128 x 256 on 8 waves, both wave groups multiply (as above); the B requests are issued by hand (see
    // load_b_chunk: 522 -> 1010 TFLOP/s symmetric, 977 -> 1063 at rho = 2, on 8192^3), and the symmetric one,
    // whose single short phase per K-step leaves a B tile little time to arrive, has a ring of three B buffers
    // (1010 -> 1042).
    // (These two carry measured factors: the issue model puts them at 0.99 and 0.96, within 8 % of the measurement,
    // but in the wrong order -- here the asymmetric tile is the faster one, by 0.4 - 3 %, and the model does not see why.)
    make_instance<Shape<128, 128, 64, 256, 2, 4, 2, 2, -1, 0, 2, 3>, true>(0.92),
    make_instance<Shape<64, 128, 64, 256, 2, 4, 4, 2>, true>(0.94),
    // 128 x 128 on a 2 x 2 grid of multiplying waves plus 4 helper waves that stage (last argument); two and
    // three workgroups per CU.  Helper waves: 920 -> 1016 TFLOP/s at 8192^3, 343-369 -> 439-514 at M = 1024, N = 2048.
    make_instance<Shape<128, 128, 64, 128, 2, 2, 2, 2, -1, 0, 2, 2, 4>, true>(),
    // (the ATB one multiplies with 16 x 16 x 32 MFMAs, compiled for 128 registers so that two workgroups still share
    // a CU: +3 % on 8192^3, +6 % at M = N = 2048; the symmetric one needs 10 registers more and loses far more to
    // spills than the MFMA form returns, so it keeps 32 x 32 x 16.  Its factor is measured, 1.08: the issue model
    // charges its second switch per K-step in full and ends 10 % low.)
    make_instance<Shape<64, 128, 64, 128, 2, 2, 4, 2, -1, 0, 2, 2, 4, 0, 16, 4>, true>(1.08),
#endif
#if ATB_IN_GROUP(2)
    // 64 x 128 with T_K = 128 (one workgroup per CU): the instance for problems with about one such tile per CU
    // (M = 1024, N = 2048: 546 - 676 TFLOP/s against 479 - 546 for the 64 x 64 tile); its ATB twin at T_MA = 32
    // measured 522 - 601 there.  Measured factor (first argument: the issue model does not describe the three
    // instances below, 0.63 / 0.96 / 0.97 against 0.83 / 1.2 / 1.24 measured): the one-round case; several rounds
    // run at 0.62 - 0.75.  A half-filled round takes as long as a full one (M = 128 and 256 at N = K = 8192: 47 and
    // 49 us), hence the cap of 1.
    make_instance<Shape<64, 64, 128, 128, 2, 2, 2, 2, -1, 0, 2, 2, 4>, true>(0.83, 1.0),
    // Small tiles for small problems: four and six workgroups per CU, with 4 and 2 helper waves (workgroups that
    // share a CU hide each other's barriers and latencies better than the issue model allows for: measured factors).
    // (several of these small workgroups share a CU, so a SIMD has several multiplying waves: MB = 16, +3-5 %)
    make_instance<Shape<64, 64, 64, 64, 2, 2, 2, 2, -1, 0, 2, 2, 4, 0, 16>, true>(1.2),
    make_instance<Shape<32, 64, 64, 64, 1, 2, 2, 2, -1, 0, 2, 2, 2, 0, 16>, true>(1.24),
    // Skinny problems (M <= 128 or so at large N, K: one or two rows of C tiles, fewer workgroups than CUs) are
    // bound by what each workgroup keeps in flight and by how fast its few waves get through a K-step, not by
    // bandwidth.  These two instances have K-steps of 256 (four times the bytes per round trip), a ring of three
    // B buffers (NB; it fits because the ATB A buffers are small, and it is what lets the symmetric 32-row tile's
    // single phase per K-step await its B tile two K-steps after the request), four helper waves next to the 1 x 2
    // grid (which alone would leave two SIMDs idle), and take the dead-row-skipping variant of the kernel body.
    // Measured at N = K = 8192 (64 x 64 x 64 tile: 72 us at every M <= 128): M <= 64: 27 - 29 us with the 32-row
    // tile (4.7 - 5.0 TB/s of B), M = 128: 39 us with the 64-row tile.  Factors from the issue model: 0.52 and 0.48
    // (measured: 0.42 - 0.49 of the fit from M = 16 to 8192).
    make_instance<Shape<32, 64, 256, 64, 1, 2, 2, 2, -1, 0, 2, 3, 4>, true>(),
    make_instance<Shape<32, 32, 256, 64, 1, 2, 2, 2, -1, 0, 2, 3, 4>, true>(),
#endif
};

}  // namespace

#if ATB_GROUP == -1
int instance_count() { return (int)(sizeof(g_instances) / sizeof(g_instances[0])); }
const Instance &instance(int i) { return g_instances[i]; }
#else
#define ATB_CAT2(a, b) a##b
#define ATB_CAT(a, b) ATB_CAT2(a, b)
// this group's slice of the table
const Instance *ATB_CAT(instances_group, ATB_GROUP)(int *n)
{
    *n = (int)(sizeof(g_instances) / sizeof(g_instances[0]));
    return g_instances;
}
#if ATB_GROUP == 0
const Instance *instances_group1(int *n);
const Instance *instances_group2(int *n);
namespace {
// the three groups' slices side by side, gathered once (no allocation: nothing here can throw)
struct InstanceTable {
    static constexpr int kMax = 32;
    Instance items[kMax];
    int count = 0;
    void append(const Instance *g, int n)
    {
        for (int i = 0; i < n && count < kMax; ++i) items[count++] = g[i];
    }
    InstanceTable()
    {
        int n = 0;
        const Instance *g = instances_group0(&n);
        append(g, n);
        g = instances_group1(&n);
        append(g, n);
        g = instances_group2(&n);
        append(g, n);
    }
};
const InstanceTable &all_instances()
{
    static const InstanceTable table;
    return table;
}
}  // namespace
int instance_count() { return all_instances().count; }
const Instance &instance(int i) { return all_instances().items[i]; }
#endif
#endif

#if ATB_GROUP == -1 || ATB_GROUP == 0
int find_instance(int T_MA, int T_MC, int T_K, int T_N)
{
    for (int i = 0; i < instance_count(); ++i) {
        const Instance &x = instance(i);
        if (x.T_MA == T_MA && x.T_MC == T_MC && x.T_K == T_K && x.T_N == T_N) return i;
    }
    return -1;
}
#endif

}  // namespace atb
