// NT matrix product on 8-bit floats for gfx950 (MI355X): C[m][n] = sum_k A[m][k] * B[n][k], A [M][K]
// and B [N][K] row-major OCP E4M3 bytes, fp32 accumulation on the matrix cores, C [M][N] in fp16 or
// bf16 (RNE).  The paper measures its matrix multiplication in FP16 and in FP8 (Section 5.2); this is
// the FP8 one.
//
// Same organisation as the 16-bit kernel: a 256 x 256 tile of C per workgroup, both operand tiles travel
// global -> LDS with direct-to-LDS loads through a ring of stages (the aref ring of Section 3.3;
// s_waitcnt vmcnt plus one s_barrier per K tile stand in for the full/empty credits), every wave copies
// its share several K tiles ahead.  The K tile is 64 elements = 64 bytes per row, so a stage has the same
// byte geometry as in the 16-bit kernel (16-row pieces of 1 KiB, row-major, the 16-byte columns of row r
// rotated by (r/4)%4), and one K tile is one k-step of the 32x32x64 MFMA (64 cycles each).
//
// Two shapes of the workgroup are compiled, and the launcher picks by K:
//   short products: 8 waves (two per SIMD), a wave owns 128 (m) x 64 (n) = 8 accumulator blocks; ring of 4
//     stages, one stage copied per tile, three tiles ahead;
//   K >= 2048: 4 waves (one per SIMD), a wave owns 128 x 128 = 16 accumulator blocks in the AGPRs; ring of 5
//     stages with PAIRED copies: a 64-byte K tile asks the L2 for half a memory line, and what limits this
//     kernel is the request path from the L2 into the CU, so two consecutive stages are copied together,
//     piece by piece, at every second tile: the two halves of a line are requested back to back and the L1
//     merges them (43 % fewer L2 requests, +6-8 % at K = 8192 ... 16384).
//
// A lane's operand of that MFMA is 32 bytes of one row.  Which 32 of the row's 64 k a lane holds does
// not matter for a sum over k as long as both operands agree: lane (row, g) takes 16-byte columns
// 2g and 2g+1 of its row of the A tile and of the B tile alike.
//
// The product is computed transposed, D = B_tile A_tile^T, so that a lane ends up with one row m of C
// and runs of four consecutive n (8-byte stores).
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

#include "gemm_launch.h"
#include "gfx950_prims.h"
#include "launch_once.h"
#include "tile_schedule.h"

namespace {

typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x8 __attribute__((ext_vector_type(8)));

// LDS requests of a tile that may still be outstanding when the next tile starts.
#ifndef GEMM8_TAIL_READS
#define GEMM8_TAIL_READS 3
#endif
// Which MFMA slots carry the copies: the odd ones (1) or the even ones (0).
#ifndef GEMM8_COPY_PHASE
#define GEMM8_COPY_PHASE 1
#endif
// Kernel configuration, fixed at compile time for the sweep harness or chosen per call by K (0):
//   1: 8 waves (two per SIMD, 128 x 64 of C each), one stage copied per tile, three tiles ahead
//   2: 8 waves, paired copies (see below)
//   3: 4 waves (one per SIMD, 128 x 128 each, a third fewer LDS reads, accumulators in the AGPRs)
//   4: 4 waves, paired copies
// Paired copies: the copies of two consecutive stages are issued together, piece by piece, at every second
// tile, so that the two 64-byte halves of a 128-byte memory line are requested back to back and the L1
// merges them into one request to the L2 (measured: 43 % fewer L2 requests); five stages, copies four and
// five tiles ahead.
#ifndef GEMM8_CONFIG
#define GEMM8_CONFIG 0
#endif
// Smallest K for which configuration 0 takes the 4-wave paired kernel (below it: 8 waves, unpaired, whose
// prologue and epilogue overlap better between the two waves of a SIMD).
constexpr int H_LARGE_K = 2048;
constexpr int H_BM = 256, H_BN = 256;   // tile of C per workgroup
constexpr int H_BK = 64;                // K tile, elements = bytes per row
#ifndef GEMM8_STAGES
#define GEMM8_STAGES 4
#endif
static_assert(GEMM8_STAGES == 4 || GEMM8_STAGES == 5, "ring protocol below");
constexpr int H_OPER_BYTES = H_BM * H_BK;            // one operand tile in the LDS (16 KiB)
constexpr int H_STAGE_BYTES = 2 * H_OPER_BYTES;      // A tile, then B tile
constexpr int H_PIECES = H_OPER_BYTES / 1024;        // 1 KiB wave-transfers per operand tile (16 rows x 64 B each)
constexpr int H_GROUP_M = 8;                         // tile rows per raster group
static_assert(H_BM == H_BN, "operand tiles are copied the same way");
constexpr int stages_of(bool paired) { return paired ? 5 : GEMM8_STAGES; }

// Logical tile -> (tile row, tile column): tile rows in groups of H_GROUP_M, a group walked column by
// column, so tiles that run at the same time share A and B row panels in the L2.
__device__ __forceinline__ void tile_coords8(int t, int ntm, int ntn, int& tm, int& tn) {
    const int per_group = H_GROUP_M * ntn;
    const int group = t / per_group, in_group = t - group * per_group;
    const int first = group * H_GROUP_M;
    const int rows = min(ntm - first, H_GROUP_M);
    tm = first + in_group % rows;
    tn = in_group / rows;
}

__device__ __forceinline__ f32x16 mfma_e4m3(i32x8 a, i32x8 b, f32x16 c) {
    // scale arguments 0: the unscaled instruction with both operands in E4M3
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 0, 0, 0, 0, 0, 0);
}

template <int OUT, int NW, bool PAIRED>
__global__ __launch_bounds__(NW * 64)
void gemm_nt_fp8_kernel(const uint8_t* __restrict__ A, const uint8_t* __restrict__ B, uint16_t* __restrict__ C,
                        int M, int N, int K, int ntm, int ntn)
{
    typedef Elem<OUT> E;
    static_assert(NW == 8 || NW == 4, "wave layout is 2 x (NW / 2)");
    constexpr int H_NB = 8 / (NW / 2);           // 32-column blocks of C per wave (its rows are 4 blocks)
    constexpr int H_STAGES = stages_of(PAIRED);
    constexpr int H_AHEAD = H_STAGES - 1;        // unpaired: copies run this many K tiles ahead of the tile being multiplied
    constexpr int H_PPW = H_PIECES / NW;         // 1 KiB pieces per wave and operand
    constexpr int H_LPG = 2 * H_PPW;             // copies a wave issues per stage
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const unsigned lds_base = (unsigned)(size_t)(LDS_AS void*)smem;

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int lr = lane & 31, g = lane >> 5;
    const int wm = wave & 1, wn = wave >> 1;          // the wave's 128 x (32 H_NB) block inside the tile

    int tm, tn;
    tile_coords8(__builtin_amdgcn_readfirstlane(tile_schedule(ntm * ntn, (int)gridDim.x, (int)blockIdx.x, 0)), ntm, ntn, tm, tn);
    const int m0 = tm * H_BM, n0 = tn * H_BN;
    const int nk = K / H_BK;
    const size_t row_bytes = (size_t)K;

    // ---- global -> LDS copies.  One copy instruction moves a 16-row piece of an operand tile (16 rows x
    // 64 B) and lane L's 16 bytes land at LDS offset 16*L.  Lanes 4r..4r+3 fetch the four 16-byte columns
    // of row r (neighbouring lanes merge into one 64-byte request); lane L fetches column
    // (L%4) ^ ((L/16)%4), which stores the columns of row r rotated by (r/4)%4 and makes the fragment
    // reads below conflict free.  Tiles that overhang the matrix clamp their rows (the surplus rows are
    // never stored).
    const bool interior = m0 + H_BM <= M && n0 + H_BN <= N;
    const int lane_row = lane >> 2, lane_col = ((lane & 3) ^ ((lane >> 4) & 3)) * 16;
    const unsigned lane_off = (unsigned)(lane_row * row_bytes) + lane_col;
    const char* a_piece[H_PPW];
    const char* b_piece[H_PPW];
    unsigned a_voff[H_PPW], b_voff[H_PPW];
#pragma unroll
    for (int i = 0; i < H_PPW; ++i) {
        const int p = wave * H_PPW + i;
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
    // One copy of stage s: piece i < H_PPW of the A tile, else piece i - H_PPW of the B tile.
    auto issue_piece = [&](int s, int i) __attribute__((always_inline)) {
        const unsigned sbase = lds_base + (s % H_STAGES) * H_STAGE_BYTES + wave * (H_PPW * 1024);
        const size_t koff = (size_t)s * H_BK;
        if (i < H_PPW) dma16(a_piece[i] + koff, a_voff[i], sbase + i * 1024);
        else dma16(b_piece[i - H_PPW] + koff, b_voff[i - H_PPW], sbase + H_OPER_BYTES + (i - H_PPW) * 1024);
    };
    auto issue_stage = [&](int s) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < H_LPG; ++i) issue_piece(s, i);
    };
    // The same for a stage that may lie past the last K tile: it then fetches the last tile again (its ring
    // slot is free by the protocol and never read), which keeps the count of copies in flight uniform.
    auto issue_piece_any = [&](int s, int i) __attribute__((always_inline)) {
        const unsigned sbase = lds_base + (s % H_STAGES) * H_STAGE_BYTES + wave * (H_PPW * 1024);
        const size_t koff = (size_t)min(s, nk - 1) * H_BK;
        if (i < H_PPW) dma16(a_piece[i] + koff, a_voff[i], sbase + i * 1024);
        else dma16(b_piece[i - H_PPW] + koff, b_voff[i - H_PPW], sbase + H_OPER_BYTES + (i - H_PPW) * 1024);
    };

    // ---- fragments: 32 rows x 64 k of an operand tile; lane l holds row l%32 and the 16-byte columns
    // 2g + h, h = 0, 1 (g = l/32), stored at position column ^ ((row/4)%4) of the row.
    int frag_lane[2];
#pragma unroll
    for (int h = 0; h < 2; ++h)
        frag_lane[h] = (lr >> 4) * 1024 + (lr & 15) * 64 + (((2 * g + h) ^ ((lr >> 2) & 3)) * 16);
    // B-matrix rows (n) feed the MFMA's A operand, A-matrix rows (m) its B operand.
    auto read_bn = [&](int s, int h, int nb) __attribute__((always_inline)) -> i32x4 {
        return *reinterpret_cast<const i32x4*>(smem + (s % H_STAGES) * H_STAGE_BYTES + frag_lane[h] + H_OPER_BYTES + (wn * H_NB + nb) * 2048);
    };
    auto read_am = [&](int s, int h, int mb) __attribute__((always_inline)) -> i32x4 {
        return *reinterpret_cast<const i32x4*>(smem + (s % H_STAGES) * H_STAGE_BYTES + frag_lane[h] + (wm * 4 + mb) * 2048);
    };

    f32x16 acc[H_NB][4];
#pragma unroll
    for (int nb = 0; nb < H_NB; ++nb)
#pragma unroll
        for (int mb = 0; mb < 4; ++mb) acc[nb][mb] = f32x16(0.f);
    // All fragments of one K tile of this wave, as 16-byte halves.
    struct TileFrags { i32x4 bn[H_NB][2]; i32x4 am[4][2]; };
    constexpr int READS_PER_TILE = 2 * (H_NB + 4), MFMAS_PER_TILE = 4 * H_NB;
    // Half-fragment request number i of a tile, in the order the MFMAs need them:
    // bn0, am0, bn1 ... bn(H_NB-1), am1, am2, am3 (MFMA q multiplies am[q / H_NB] with bn[q % H_NB]).
    auto read_half = [&](TileFrags& t, int s, int i) __attribute__((always_inline)) {
        const int f = i >> 1, h = i & 1;
        if (f == 0) t.bn[0][h] = read_bn(s, h, 0);
        else if (f == 1) t.am[0][h] = read_am(s, h, 0);
        else if (f <= H_NB) t.bn[f - 1][h] = read_bn(s, h, f - 1);
        else t.am[f - H_NB][h] = read_am(s, h, f - H_NB);
    };
    auto whole = [](const i32x4 (&x)[2]) __attribute__((always_inline)) -> i32x8 {
        return __builtin_shufflevector(x[0], x[1], 0, 1, 2, 3, 4, 5, 6, 7);
    };
    // Slot plan of `tile`: a copy behind every second MFMA, the requests spread evenly over all slots
    // (the slots that carry a copy take the smaller share).
    constexpr int READS_LO = READS_PER_TILE / MFMAS_PER_TILE, READS_HI = (READS_PER_TILE + MFMAS_PER_TILE - 1) / MFMAS_PER_TILE;
    static_assert(H_LPG * 2 == MFMAS_PER_TILE && (READS_LO + READS_HI) * (MFMAS_PER_TILE / 2) == READS_PER_TILE, "slot plan of `tile`");

    if constexpr (PAIRED) {
    // ---- paired copies.  Ring of five stages.  At the barrier of an even tile e the slots of stages e - 1
    // and e are free (the fragments of tile e were read during tile e - 1, and every wave waited for its
    // requests before the barrier), and the wave issues its pieces of stages e + 4 and e + 5 alternately,
    // one behind each MFMA of the tile; odd tiles issue none.  Before barrier j a wave has waited for its own
    // copies of stage j + 1: what may still be in flight is the pair issued two tiles ago (j even), or the
    // last piece of stage j + 2 and the pair issued one tile ago (j odd).
    static_assert(2 * H_LPG == MFMAS_PER_TILE, "one copy behind each MFMA of an even tile");
#pragma unroll
    for (int s0 = 0; s0 < 4; ++s0)
#pragma unroll
        for (int i = 0; i < H_LPG; ++i) issue_piece_any(s0, i);
    wait_vmcnt<3 * H_LPG>();                  // stage 0
    __builtin_amdgcn_s_barrier();
    auto tile2 = [&](int j, const TileFrags& cur, TileFrags& nxt, auto even_tag) __attribute__((always_inline)) {
        constexpr bool EVEN = decltype(even_tag)::value;
        if (EVEN) wait_vmcnt<2 * H_LPG>(); else wait_vmcnt<2 * H_LPG + 1>();
        __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0): this wave's reads of stage j are complete
        __builtin_amdgcn_s_barrier();
        const int jn = min(j + 1, nk - 1);    // (the last tile re-reads itself: harmless, unused)
        int next_read = 0;
#pragma unroll
        for (int q = 0; q < MFMAS_PER_TILE; ++q) {
            const int mb = q / H_NB, nb = q % H_NB;
            acc[nb][mb] = mfma_e4m3(whole(cur.bn[nb]), whole(cur.am[mb]), acc[nb][mb]);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int r = 0; r < ((q & 1) ? READS_LO : READS_HI); ++r) read_half(nxt, jn, next_read++);
            if (EVEN) issue_piece_any(j + 4 + (q & 1), q >> 1);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    TileFrags X, Y;
#pragma unroll
    for (int i = 0; i < READS_PER_TILE; ++i) read_half(X, 0, i);
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
    // Own copies of stage j+1 complete: only the stages after it stay in flight.
    auto wait_next_stage = [&](int j) __attribute__((always_inline)) {
        if (H_AHEAD > 3 && j + 3 < nk) wait_vmcnt<2 * H_LPG>();
        else if (j + 2 < nk) wait_vmcnt<H_LPG>();
        else wait_vmcnt<0>();
    };

    // ---- prologue: H_AHEAD stages in flight; stage 0 complete for everyone; first fragments requested
    issue_stage(0);
    if (nk > 1) issue_stage(1);
    if (nk > 2) issue_stage(2);
    if (H_AHEAD > 3 && nk > 3) issue_stage(3);
    if (H_AHEAD > 3 && nk > 3) wait_vmcnt<3 * H_LPG>();
    else if (nk > 2) wait_vmcnt<2 * H_LPG>(); else if (nk > 1) wait_vmcnt<H_LPG>(); else wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();

    // One K tile: 8 MFMAs (16 with four waves) on the fragments in `cur` (requested during the previous
    // tile).  Behind each MFMA go requests for the next tile's fragments into `nxt` and, behind every second
    // one, a copy of the stage three tiles ahead: 12 LDS requests and 4 copies over 8 slots of 64 cycles
    // (16 and 8 over 16).  Stage j+1 is
    // complete at barrier j, which makes the early requests legal.
    auto tile = [&](int j, const TileFrags& cur, TileFrags& nxt, auto steady_tag) __attribute__((always_inline)) {
        constexpr bool STEADY = decltype(steady_tag)::value;   // j + H_AHEAD < nk is known: no tests in the tile
        if (STEADY) wait_vmcnt<(H_AHEAD - 2) * H_LPG>(); else wait_next_stage(j);
        __builtin_amdgcn_s_barrier();
        const int cs = STEADY || j + H_AHEAD < nk ? j + H_AHEAD : -1;   // the stage whose copies go out during this tile
        const int jn = STEADY || j + 1 < nk ? j + 1 : j;                // (the last tile re-reads itself: harmless, unused)
        int next_read = 0;
#pragma unroll
        for (int q = 0; q < MFMAS_PER_TILE; ++q) {
            const int mb = q / H_NB, nb = q % H_NB;
            acc[nb][mb] = mfma_e4m3(whole(cur.bn[nb]), whole(cur.am[mb]), acc[nb][mb]);
            __builtin_amdgcn_sched_barrier(0);
            const bool copy_slot = (q & 1) == GEMM8_COPY_PHASE;
#pragma unroll
            for (int r = 0; r < (copy_slot ? READS_LO : READS_HI); ++r) read_half(nxt, jn, next_read++);
            if (copy_slot && (STEADY || cs >= 0)) issue_piece(cs, q >> 1);
            __builtin_amdgcn_sched_barrier(0);
        }
        // The fragments the next tile needs first were requested first and have landed; the last few
        // requests may still be in flight.  Saying so here keeps the compiler from waiting for ALL
        // outstanding requests at the loop top.
        __builtin_amdgcn_s_waitcnt(0xC07F | (GEMM8_TAIL_READS << 8));   // lgkmcnt(GEMM8_TAIL_READS)
    };

    TileFrags X, Y;
#pragma unroll
    for (int i = 0; i < READS_PER_TILE; ++i) read_half(X, 0, i);
    __builtin_amdgcn_s_waitcnt(0xC07F);       // lgkmcnt(0)
    // Tiles in pairs so that the two fragment sets swap roles without a register copy; bottom-tested
    // loops, an odd last tile peeled off.  While a tile H_AHEAD ahead exists ("steady") a tile body has
    // no tests at all; the last H_AHEAD tiles and short products take the body that tests what is left
    // to copy and to wait for (a wave-uniform branch around every copy costs 2 % at K = 8192).
    typedef std::integral_constant<bool, true> steady_t;
    typedef std::integral_constant<bool, false> draining_t;
    int j = 0;
    if (nk >= H_AHEAD + 2) {
        do {
            tile(j, X, Y, steady_t());
            tile(j + 1, Y, X, steady_t());
            j += 2;
        } while (j + 1 + H_AHEAD < nk);
    }
    if (j + 1 < nk) {
        do {
            tile(j, X, Y, draining_t());
            tile(j + 1, Y, X, draining_t());
            j += 2;
        } while (j + 1 < nk);
    }
    if (j < nk) tile(j, X, Y, draining_t());

    }  // !PAIRED

    // ---- epilogue: lane holds row m of C and, per accumulator register quad, four consecutive n
    const bool vec_ok = (N & 3) == 0 && (reinterpret_cast<uintptr_t>(C) & 7) == 0;
#pragma unroll
    for (int mb = 0; mb < 4; ++mb) {
        const int m = m0 + wm * 128 + mb * 32 + lr;
        if (m >= M) continue;
        uint16_t* crow = C + (size_t)m * N;
#pragma unroll
        for (int nb = 0; nb < H_NB; ++nb)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                const int n = n0 + wn * (H_NB * 32) + nb * 32 + i4 * 8 + g * 4;
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

template <int OUT, int NW, bool PAIRED>
int launch8(const GemmLaunchArgs& a)
{
    constexpr int smem = stages_of(PAIRED) * H_STAGE_BYTES;
    auto kern = gemm_nt_fp8_kernel<OUT, NW, PAIRED>;
    static PerDeviceOnce once;                  // the attribute belongs to the (kernel, device) pair
    if (once.prepare(reinterpret_cast<const void*>(kern), smem) < 0) return -1;
    const uint8_t* A = (const uint8_t*)a.a;
    const uint8_t* B = (const uint8_t*)a.b;
    uint16_t* C = (uint16_t*)a.c;
    int M = a.M, N = a.N, K = a.K;
    int ntm = (M + H_BM - 1) / H_BM, ntn = (N + H_BN - 1) / H_BN;
    void* args[] = {&A, &B, &C, &M, &N, &K, &ntm, &ntn};
    const hipError_t e = hipLaunchKernel(reinterpret_cast<const void*>(kern), dim3((unsigned)(ntm * ntn)), dim3(NW * 64),
                                         args, smem, (hipStream_t)a.stream);
    return e == hipSuccess ? 0 : -1;
}

int config_for(int K) { return GEMM8_CONFIG != 0 ? GEMM8_CONFIG : (K >= H_LARGE_K ? 4 : 1); }

template <int OUT>
int launch8_out(const GemmLaunchArgs& a)
{
    switch (a.config != 0 ? a.config : config_for(a.K)) {
        case 1: return launch8<OUT, 8, false>(a);
        case 2: return launch8<OUT, 8, true>(a);
        case 3: return launch8<OUT, 4, false>(a);
        default: return launch8<OUT, 4, true>(a);
    }
}

}  // namespace

int gemm_fp8_launch(const GemmLaunchArgs& a) { return a.dtype == 0 ? launch8_out<0>(a) : launch8_out<1>(a); }

// Reported for the configuration a large K takes.
int gemm_fp8_launch_tile_param(int which)
{
    const int cfg = config_for(1 << 20);
    switch (which) {
        case 0: return H_BM;
        case 1: return H_BN;
        case 2: return H_BK;
        case 3: return stages_of(cfg == 2 || cfg == 4);
        case 4: return (cfg >= 3 ? 4 : 8) * 64;
        default: return -1;
    }
}
