// NT matrix product for gfx950 (MI355X): C[m][n] = sum_k A[m][k] * B[n][k], A [M][K] and B [N][K]
// row-major 16-bit, fp32 accumulation on the matrix cores, C [M][N] in the input type (RNE).
//
// This is the paper's other headline kernel (the matrix multiplication of Sections 3.1 and 5.2) on
// the same machinery as the attention kernel: both operand tiles travel global -> LDS with
// direct-to-LDS loads through a ring of stages (the aref ring of Section 3.3; s_waitcnt vmcnt plus one
// s_barrier per K tile stand in for the full/empty credits), and the 32x32x16 MFMA consumes them.
// There is no producer wave: every wave issues its share of the copies several K tiles ahead and computes.
//
// Workgroup: a 256 x 256 tile of C, by 8 waves (two per SIMD; a wave owns 128 (m) x 64 (n), 8 accumulator
// blocks) or by 4 waves (one per SIMD; 128 x 128, 16 accumulator blocks in the AGPRs).  The product is
// computed transposed, D = B_tile A_tile^T, so that a lane ends up with one row m of C and runs of four
// consecutive n: the 16-bit results leave as 8-byte stores (computed the other way round a lane would
// hold single elements of 16 different rows).
//
// Schedule of one wave, K tile j (32 wide, two MFMA k-steps): wait for its own copies of stage j+1;
// barrier; then the MFMAs on fragments that were requested during tile j-1, with LDS requests (fragments
// of tile j+1) and copies issued one at a time behind the MFMAs.  Which copies:
//   unpaired (ring of 4): the pieces of stage j+3, whose slot tile j-1 has just released;
//   paired (ring of 5): a K tile is 64 bytes per row, half a memory line, and the limit of this kernel is
//   the request path from the L2 into the CU; so even tiles issue the pieces of stages j+4 and j+5
//   alternately and odd tiles none: the two halves of a line are requested back to back and the L1 merges
//   them into one request to the L2 (+9-13 % at K >= 2048).
// The launcher takes the 4-wave paired kernel from K = 2048 on and the 8-wave paired kernel below.
//
// Measured on the device (M = N = 8192, K = 8192, fp16 N(0,1) operands, same box and session), 8 waves,
// unpaired: 1.16 PFLOP/s; with the copies left out (wrong results, timing only) 1.40; with the
//   fragment reads left out 1.23; with neither 1.60, which is the chip's random-operand MFMA-only
//   rate.  Copies always taken from the same K tile (L2 hits only): no change, so the HBM side is
//   not the limit.  Four extra producer waves that do all the copying (warp specialisation as in the
//   paper; tried with a leaner fragment schedule that fits the 168 registers of three waves per SIMD):
//   slower, 1.00.  A fifth ring stage without pairing: the same.  Lanes of a copy
//   mapped to rows (lane -> row L%16) instead of to the 16-byte columns of a row: 0.96.
// All four configurations, same session: 1.17 (8 waves), 1.28 (8, paired), 1.22 (4 waves), 1.30 (4, paired).
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

#include "gemm_launch.h"
#include "gfx950_prims.h"
#include "launch_once.h"
#include "tile_schedule.h"

namespace {

#ifdef GEMM_TIMING
// Profiling builds only: per-wave cycle totals of the main-loop sections of the first workgroups.
__device__ unsigned long long gemm_dbg[256 * 8 * 8];
#define GSTAMP(var) unsigned long long var; __builtin_amdgcn_sched_barrier(0); \
    asm volatile("s_memtime %0\n\ts_waitcnt lgkmcnt(0)" : "=s"(var) :: "memory"); __builtin_amdgcn_sched_barrier(0)
#define GACC(slot, a, b) dbg_acc[slot] += (b) - (a)
#else
#define GSTAMP(var)
#define GACC(slot, a, b)
#endif

// LDS requests of a tile that may still be outstanding when the next tile starts (see the end of `tile`).
#ifndef GEMM_TAIL_READS
#define GEMM_TAIL_READS 3
#endif
// Kernel configuration, fixed at compile time for the sweep harness or chosen per call by K (0):
//   1: 8 waves (two per SIMD, 128 x 64 of C each), one stage copied per tile, three tiles ahead
//   2: 8 waves, paired copies
//   3: 4 waves (one per SIMD, 128 x 128 each, a third fewer LDS reads, accumulators in the AGPRs)
//   4: 4 waves, paired copies
// Paired copies: a 32-element K tile is 64 bytes per row, half a memory line, and what limits this kernel
// is the request path from the L2 into the CU.  The copies of two consecutive stages are therefore issued
// together, piece by piece, at every second tile: the two halves of a line are requested back to back and
// the L1 merges them into one request to the L2.  Five stages, copies four and five tiles ahead.
#ifndef GEMM_CONFIG
#define GEMM_CONFIG 0
#endif
// Configuration 0: the 4-wave paired kernel from this K on, the 8-wave paired kernel below it (whose
// prologue and epilogue overlap better between the two waves of a SIMD).
constexpr int G_LARGE_K = 2048;
constexpr int G_BM = 256, G_BN = 256;   // tile of C per workgroup
constexpr int G_BK = 32;                // K tile
#ifndef GEMM_STAGES
#define GEMM_STAGES 4
#endif
static_assert(GEMM_STAGES == 4 || GEMM_STAGES == 5, "ring protocol below");
constexpr int G_OPER_BYTES = G_BM * G_BK * 2;        // one operand tile in the LDS (16 KiB)
constexpr int G_STAGE_BYTES = 2 * G_OPER_BYTES;      // A tile, then B tile
constexpr int G_PIECES = G_OPER_BYTES / 1024;        // 1 KiB wave-transfers per operand tile (16 rows x 64 B each)
constexpr int G_GROUP_M = 8;                         // tile rows per raster group (see tile_coords)
static_assert(G_BM == G_BN, "operand tiles are copied the same way");
constexpr int g_stages_of(bool paired) { return paired ? 5 : GEMM_STAGES; }

// Logical tile -> (tile row, tile column): tile rows are taken in groups of G_GROUP_M and a group is
// walked column by column, so tiles that run at the same time share A row panels and B row panels
// in the L2 (the usual grouped ordering of a tiled matrix product).
__device__ __forceinline__ void tile_coords(int t, int ntm, int ntn, int& tm, int& tn) {
    const int per_group = G_GROUP_M * ntn;
    const int group = t / per_group, in_group = t - group * per_group;
    const int first = group * G_GROUP_M;
    const int rows = min(ntm - first, G_GROUP_M);
    tm = first + in_group % rows;
    tn = in_group / rows;
}

template <int DTYPE, int NW, bool PAIRED>
__global__ __launch_bounds__(NW * 64)
void gemm_nt_kernel(const uint16_t* __restrict__ A, const uint16_t* __restrict__ B, uint16_t* __restrict__ C,
                    int M, int N, int K, int ntm, int ntn)
{
    typedef Elem<DTYPE> E;
    static_assert(NW == 8 || NW == 4, "wave layout is 2 x (NW / 2)");
    constexpr int G_CW = NW;                     // waves per workgroup: every wave copies and computes
    constexpr int G_NB = 8 / (NW / 2);           // 32-column blocks of C per wave (the wave's rows are always 4 blocks)
    constexpr int G_STAGES = g_stages_of(PAIRED);
    constexpr int G_AHEAD = G_STAGES - 1;        // unpaired: copies run this many K tiles ahead of the tile being multiplied
    constexpr int G_PPW = G_PIECES / NW;         // 1 KiB pieces per wave and operand
    constexpr int G_LPG = 2 * G_PPW;             // copies a wave issues per stage
    static_assert(4 * G_LPG <= 63, "the stages in flight must fit the vmcnt counter");
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const unsigned lds_base = (unsigned)(size_t)(LDS_AS void*)smem;

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int lr = lane & 31, g = lane >> 5;
    const int wm = wave & 1, wn = (wave >> 1) & (G_CW / 2 - 1);   // the wave's 128 x (32 G_NB) block inside the tile

    int tm, tn;
    tile_coords(__builtin_amdgcn_readfirstlane(tile_schedule(ntm * ntn, (int)gridDim.x, (int)blockIdx.x, 0)), ntm, ntn, tm, tn);
    const int m0 = tm * G_BM, n0 = tn * G_BN;
    const int nk = K / G_BK;
    const size_t row_bytes = (size_t)K * 2;

    // ---- global -> LDS copies.  One copy instruction moves a 16-row block of an operand tile (16 rows x
    // 64 B = 1 KiB) and lane L's 16 bytes land at LDS offset 16*L, so the lane -> address map fixes the
    // LDS layout.  Lanes 4r..4r+3 fetch the four 16-byte columns of row r: only neighbouring lanes are
    // merged into one 64-byte request on the way to the L2 (measured: 29 TB/s chip-wide against 9.5 with
    // lane -> row L%16).  The block is therefore row-major in the LDS, 64 B per row, which alone would
    // put rows r and r+4 on the same banks for the fragment reads below; the columns of row r are
    // stored rotated by (r/4)%4 (lane L fetches column (L%4) ^ ((L/16)%4)), which makes them conflict free.
    // Inside the matrix the per-lane offset is a constant and the piece / K-tile offset sits in the scalar
    // base; tiles that overhang the matrix clamp their rows (the surplus rows are never stored).
    const bool interior = m0 + G_BM <= M && n0 + G_BN <= N;
    const int lane_row = lane >> 2, lane_col = ((lane & 3) ^ ((lane >> 4) & 3)) * 16;
    const unsigned lane_off = (unsigned)(lane_row * row_bytes) + lane_col;
    const char* a_piece[G_PPW];
    const char* b_piece[G_PPW];
    unsigned a_voff[G_PPW], b_voff[G_PPW];
#pragma unroll
    for (int i = 0; i < G_PPW; ++i) {
        const int p = wave * G_PPW + i;
        if (interior) {
            a_piece[i] = reinterpret_cast<const char*>(A) + (size_t)(m0 + p * 16) * row_bytes;
            b_piece[i] = reinterpret_cast<const char*>(B) + (size_t)(n0 + p * 16) * row_bytes;
            a_voff[i] = b_voff[i] = lane_off;
        } else {
            a_piece[i] = reinterpret_cast<const char*>(A);
            b_piece[i] = reinterpret_cast<const char*>(B);
            a_voff[i] = (unsigned)((size_t)min(m0 + p * 16 + lane_row, M - 1) * row_bytes) + lane_col;
            b_voff[i] = (unsigned)((size_t)min(n0 + p * 16 + lane_row, N - 1) * row_bytes) + lane_col;
        }
    }
    // One copy of stage s: piece i < G_PPW of the A tile, else piece i - G_PPW of the B tile.
    auto issue_piece = [&](int s, int i) __attribute__((always_inline)) {
        const unsigned sbase = lds_base + (s % G_STAGES) * G_STAGE_BYTES + wave * (G_PPW * 1024);
        const size_t koff = (size_t)s * (G_BK * 2);
        if (i < G_PPW) dma16(a_piece[i] + koff, a_voff[i], sbase + i * 1024);
        else dma16(b_piece[i - G_PPW] + koff, b_voff[i - G_PPW], sbase + G_OPER_BYTES + (i - G_PPW) * 1024);
    };
    auto issue_stage = [&](int s) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < G_LPG; ++i) issue_piece(s, i);
    };
    // The same for a stage that may lie past the last K tile: it then fetches the last tile again (its ring
    // slot is free by the protocol and never read), which keeps the count of copies in flight uniform.
    auto issue_piece_any = [&](int s, int i) __attribute__((always_inline)) {
        const unsigned sbase = lds_base + (s % G_STAGES) * G_STAGE_BYTES + wave * (G_PPW * 1024);
        const size_t koff = (size_t)min(s, nk - 1) * (G_BK * 2);
        if (i < G_PPW) dma16(a_piece[i] + koff, a_voff[i], sbase + i * 1024);
        else dma16(b_piece[i - G_PPW] + koff, b_voff[i - G_PPW], sbase + G_OPER_BYTES + (i - G_PPW) * 1024);
    };

    // ---- fragments: 32 rows x 16 k of an operand tile; lane l holds row l%32, k = 16*ks + 8*(l/32) .. +7
    // (row lr%16 of 16-row block lr/16; 16-byte column 2*ks + g, stored at position column ^ ((row/4)%4))
    int frag_lane[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
        frag_lane[ks] = (lr >> 4) * 1024 + (lr & 15) * 64 + (((ks * 2 + g) ^ ((lr >> 2) & 3)) * 16);
    // B-matrix rows (n) feed the MFMA's A operand, A-matrix rows (m) its B operand.
    auto read_bn = [&](int s, int ks, int nb) __attribute__((always_inline)) -> s16x8 {
        return *reinterpret_cast<const s16x8*>(smem + (s % G_STAGES) * G_STAGE_BYTES + frag_lane[ks] + G_OPER_BYTES + (wn * G_NB + nb) * 2048);
    };
    auto read_am = [&](int s, int ks, int mb) __attribute__((always_inline)) -> s16x8 {
        return *reinterpret_cast<const s16x8*>(smem + (s % G_STAGES) * G_STAGE_BYTES + frag_lane[ks] + (wm * 4 + mb) * 2048);
    };

    f32x16 acc[G_NB][4];
#pragma unroll
    for (int nb = 0; nb < G_NB; ++nb)
#pragma unroll
        for (int mb = 0; mb < 4; ++mb) acc[nb][mb] = f32x16(0.f);
    // All fragments of one K tile of this wave: 2 k-steps x (G_NB B-matrix + 4 A-matrix fragments).
    struct TileFrags { s16x8 bn[2][G_NB]; s16x8 am[2][4]; };
    constexpr int FRAGS_PER_TILE = 2 * (G_NB + 4), MFMAS_PER_TILE = 8 * G_NB;
    // Fragment number i of a tile, in the order the MFMAs need them.
    auto read_frag = [&](TileFrags& t, int s, int i) __attribute__((always_inline)) {
        const int ks = i / (G_NB + 4), r = i % (G_NB + 4);
        if (r < G_NB) t.bn[ks][r] = read_bn(s, ks, r);
        else t.am[ks][r - G_NB] = read_am(s, ks, r - G_NB);
    };
    static_assert(FRAGS_PER_TILE + G_LPG <= MFMAS_PER_TILE, "one request or copy per MFMA slot");

    if constexpr (PAIRED) {
    // ---- paired copies.  Ring of five stages.  At the barrier of an even tile e the slots of stages e - 1
    // and e are free (the fragments of tile e were read during tile e - 1, and every wave waited for its
    // requests before the barrier), and the wave issues its pieces of stages e + 4 and e + 5 alternately,
    // one behind every second MFMA of the tile; odd tiles issue none.  Before barrier j a wave has waited for
    // its own copies of stage j + 1: what may still be in flight is the pair issued two tiles ago (j even),
    // or the last piece of stage j + 2 and the pair issued one tile ago (j odd).
    static_assert(4 * G_LPG == MFMAS_PER_TILE, "one copy behind every second MFMA of an even tile");
#pragma unroll
    for (int s0 = 0; s0 < 4; ++s0)
#pragma unroll
        for (int i = 0; i < G_LPG; ++i) issue_piece_any(s0, i);
    wait_vmcnt<3 * G_LPG>();                  // stage 0
    __builtin_amdgcn_s_barrier();
    auto tile2 = [&](int j, const TileFrags& cur, TileFrags& nxt, auto even_tag) __attribute__((always_inline)) {
        constexpr bool EVEN = decltype(even_tag)::value;
        if (EVEN) wait_vmcnt<2 * G_LPG>(); else wait_vmcnt<2 * G_LPG + 1>();
        __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0): this wave's reads of stage j are complete
        __builtin_amdgcn_s_barrier();
        const int jn = min(j + 1, nk - 1);    // (the last tile re-reads itself: harmless, unused)
        int next_frag = 0;
#pragma unroll
        for (int q = 0; q < MFMAS_PER_TILE; ++q) {
            const int ks = q / (4 * G_NB), mb = (q / G_NB) % 4, nb = q % G_NB;
            acc[nb][mb] = E::mfma(cur.bn[ks][nb], cur.am[ks][mb], acc[nb][mb]);
            __builtin_amdgcn_sched_barrier(0);
            // requests behind the even MFMAs and, while some are left, behind every fourth odd one
            if (next_frag < FRAGS_PER_TILE && ((q & 1) == 0 || (q & 3) == 1)) {
                read_frag(nxt, jn, next_frag);
                ++next_frag;
            }
            if (EVEN && (q & 1)) issue_piece_any(j + 4 + ((q >> 1) & 1), q >> 2);
            __builtin_amdgcn_sched_barrier(0);
        }
        static_assert(FRAGS_PER_TILE <= MFMAS_PER_TILE / 2 + MFMAS_PER_TILE / 4, "every fragment has a slot");
    };
    TileFrags X, Y;
#pragma unroll
    for (int i = 0; i < FRAGS_PER_TILE; ++i) read_frag(X, 0, i);
    {
        typedef std::integral_constant<bool, true> even_t;
        typedef std::integral_constant<bool, false> odd_t;
        int j = 0;
        if (nk >= 2) {
            do {
                tile2(j, X, Y, even_t());
                tile2(j + 1, Y, X, odd_t());
                j += 2;
            } while (j + 1 < nk);
        }
        if (j < nk) tile2(j, X, Y, even_t());
    }
    wait_vmcnt<0>();                          // surplus copies past the last tile
    } else {
    // Own copies of stage j+1 complete: only the stages after it (at most G_AHEAD - 2 of them) stay in flight.
    auto wait_next_stage = [&](int j) __attribute__((always_inline)) {
        if (G_AHEAD > 3 && j + 3 < nk) wait_vmcnt<2 * G_LPG>();
        else if (j + 2 < nk) wait_vmcnt<G_LPG>();
        else wait_vmcnt<0>();
    };

    // ---- prologue: G_AHEAD stages in flight; stage 0 complete for everyone; first fragments requested
    issue_stage(0);
    if (nk > 1) issue_stage(1);
    if (nk > 2) issue_stage(2);
    if (G_AHEAD > 3 && nk > 3) issue_stage(3);
    // stage 0 must be complete: everything but the later stages' copies
    if (G_AHEAD > 3 && nk > 3) wait_vmcnt<3 * G_LPG>();
    else if (nk > 2) wait_vmcnt<2 * G_LPG>(); else if (nk > 1) wait_vmcnt<G_LPG>(); else wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();

    // One K tile: multiply from the fragments in `cur` (requested during the previous tile) and request
    // the next tile's fragments into `nxt`, one request after each MFMA: with the copies' writes the LDS
    // is close to saturated and a request can take hundreds of cycles, so every fragment gets a whole
    // tile (16 MFMAs per wave, 32 per SIMD) to arrive.  Stage j+1 is complete at barrier j, which is what
    // makes the early requests legal, and the matrix core has work the moment the barrier opens.  When
    // every wave copies, the copies of the stage three tiles ahead go out in the remaining MFMA slots,
    // evenly spread: a wave queueing for the CU's copy path cannot issue its MFMAs meanwhile.
#ifdef GEMM_TIMING
    unsigned long long dbg_acc[8] = {};
    const unsigned long long rt0 = __builtin_amdgcn_s_memrealtime(), ct0 = __builtin_readcyclecounter();
#endif
    auto tile = [&](int j, const TileFrags& cur, TileFrags& nxt, auto steady_tag) __attribute__((always_inline)) {
        constexpr bool STEADY = decltype(steady_tag)::value;   // j + G_AHEAD < nk is known: no tests in the tile
        GSTAMP(t0);
        if (STEADY) wait_vmcnt<(G_AHEAD - 2) * G_LPG>(); else wait_next_stage(j);
        GSTAMP(t1);
        __builtin_amdgcn_s_barrier();
        GSTAMP(t2);
        const int cs = STEADY || j + G_AHEAD < nk ? j + G_AHEAD : -1;   // the stage whose copies go out during this tile
        const int jn = STEADY || j + 1 < nk ? j + 1 : j;                // (the last tile re-reads itself: harmless, unused)
        constexpr int COPY_EVERY = MFMAS_PER_TILE / G_LPG;
        int next_frag = 0;
#pragma unroll
        for (int q = 0; q < MFMAS_PER_TILE; ++q) {
            const int ks = q / (4 * G_NB), mb = (q / G_NB) % 4, nb = q % G_NB;
            acc[nb][mb] = E::mfma(cur.bn[ks][nb], cur.am[ks][mb], acc[nb][mb]);
            __builtin_amdgcn_sched_barrier(0);
            if (q % COPY_EVERY == COPY_EVERY - 1) {
                if (STEADY || cs >= 0) issue_piece(cs, q / COPY_EVERY);
            } else if (next_frag < FRAGS_PER_TILE) {
                read_frag(nxt, jn, next_frag);
                ++next_frag;
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        GSTAMP(t5);
        GACC(0, t0, t1); GACC(1, t1, t2); GACC(4, t2, t5);
        // The fragments the next tile needs first were requested first and have landed; the last few
        // requests may still be in flight (their MFMAs come late in the next tile).  Saying so here, instead
        // of nothing, keeps the compiler from waiting for ALL outstanding requests at the loop top, and
        // waiting for all of them would stall every tile by an LDS latency.
        __builtin_amdgcn_s_waitcnt(0xC07F | (GEMM_TAIL_READS << 8));   // lgkmcnt(GEMM_TAIL_READS)
    };

    TileFrags X, Y;
#pragma unroll
    for (int i = 0; i < FRAGS_PER_TILE; ++i) read_frag(X, 0, i);
    __builtin_amdgcn_s_waitcnt(0xC07F);       // lgkmcnt(0)
    // Tiles are taken in pairs so that the two fragment sets swap roles without a register copy; the
    // loops are bottom-tested (with the exit test at the top the accumulators would be copied every
    // iteration) and an odd last tile is peeled off.  While a tile G_AHEAD ahead exists ("steady") a
    // tile body has no tests at all; the last G_AHEAD tiles and short products take the body that tests
    // what is left to copy and to wait for.
    typedef std::integral_constant<bool, true> steady_t;
    typedef std::integral_constant<bool, false> draining_t;
    int j = 0;
    if (nk >= G_AHEAD + 2) {
        do {
            tile(j, X, Y, steady_t());
            tile(j + 1, Y, X, steady_t());
            j += 2;
        } while (j + 1 + G_AHEAD < nk);
    }
    if (j + 1 < nk) {
        do {
            tile(j, X, Y, draining_t());
            tile(j + 1, Y, X, draining_t());
            j += 2;
        } while (j + 1 < nk);
    }
    if (j < nk) tile(j, X, Y, draining_t());

#ifdef GEMM_TIMING
    if (blockIdx.x < 256 && lane == 0) {
        dbg_acc[5] = nk;
        dbg_acc[6] = __builtin_amdgcn_s_memrealtime() - rt0;
        dbg_acc[7] = __builtin_readcyclecounter() - ct0;
        for (int i = 0; i < 8; ++i) gemm_dbg[(blockIdx.x * 8 + wave) * 8 + i] = dbg_acc[i];
    }
#endif
    }  // !PAIRED
    // ---- epilogue: lane holds row m of C and, per accumulator register quad, four consecutive n
    const bool vec_ok = (N & 3) == 0 && (reinterpret_cast<uintptr_t>(C) & 7) == 0;
#pragma unroll
    for (int mb = 0; mb < 4; ++mb) {
        const int m = m0 + wm * 128 + mb * 32 + lr;
        if (m >= M) continue;
        uint16_t* crow = C + (size_t)m * N;
#pragma unroll
        for (int nb = 0; nb < G_NB; ++nb)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                const int n = n0 + wn * (G_NB * 32) + nb * 32 + i4 * 8 + g * 4;
                u32x2 w;
                w[0] = E::pack2(acc[nb][mb][i4 * 4 + 0], acc[nb][mb][i4 * 4 + 1]);
                w[1] = E::pack2(acc[nb][mb][i4 * 4 + 2], acc[nb][mb][i4 * 4 + 3]);
                if (vec_ok && n + 3 < N) {
                    *reinterpret_cast<u32x2*>(crow + n) = w;
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (n + e < N) crow[n + e] = (uint16_t)(w[e >> 1] >> ((e & 1) * 16));
                }
            }
    }
}

template <int DTYPE, int NW, bool PAIRED>
int launch(const GemmLaunchArgs& a)
{
    constexpr int smem = g_stages_of(PAIRED) * G_STAGE_BYTES;
    auto kern = gemm_nt_kernel<DTYPE, NW, PAIRED>;
    static PerDeviceOnce once;                  // the attribute belongs to the (kernel, device) pair
    if (once.prepare(reinterpret_cast<const void*>(kern), smem) < 0) return -1;
    const uint16_t* A = (const uint16_t*)a.a;
    const uint16_t* B = (const uint16_t*)a.b;
    uint16_t* C = (uint16_t*)a.c;
    int M = a.M, N = a.N, K = a.K;
    int ntm = (M + G_BM - 1) / G_BM, ntn = (N + G_BN - 1) / G_BN;
    void* args[] = {&A, &B, &C, &M, &N, &K, &ntm, &ntn};
    const hipError_t e = hipLaunchKernel(reinterpret_cast<const void*>(kern), dim3((unsigned)(ntm * ntn)), dim3(NW * 64),
                                         args, smem, (hipStream_t)a.stream);
    return e == hipSuccess ? 0 : -1;
}

int config_for(int K) { return GEMM_CONFIG != 0 ? GEMM_CONFIG : (K >= G_LARGE_K ? 4 : 2); }

template <int DTYPE>
int launch_dtype(const GemmLaunchArgs& a)
{
    switch (a.config != 0 ? a.config : config_for(a.K)) {
        case 1: return launch<DTYPE, 8, false>(a);
        case 2: return launch<DTYPE, 8, true>(a);
        case 3: return launch<DTYPE, 4, false>(a);
        default: return launch<DTYPE, 4, true>(a);
    }
}

}  // namespace

#ifdef GEMM_TIMING
extern "C" int gemm_dbg_read(unsigned long long* host, int n)
{
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(gemm_dbg), sizeof(unsigned long long) * n);
}
#endif

int gemm_launch(const GemmLaunchArgs& a) { return a.dtype == 0 ? launch_dtype<0>(a) : launch_dtype<1>(a); }

// Reported for the configuration a large K takes.
int gemm_launch_tile_param(int which)
{
    const int cfg = config_for(1 << 20);
    switch (which) {
        case 0: return G_BM;
        case 1: return G_BN;
        case 2: return G_BK;
        case 3: return g_stages_of(cfg == 2 || cfg == 4);
        case 4: return (cfg >= 3 ? 4 : 8) * 64;
        default: return -1;
    }
}
