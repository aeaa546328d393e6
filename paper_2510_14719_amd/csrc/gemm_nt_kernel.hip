// NT matrix product for gfx950 (MI355X): C[m][n] = sum_k A[m][k] * B[n][k], A [M][K] and B [N][K]
// row-major 16-bit, fp32 accumulation on the matrix cores, C [M][N] in the input type (RNE).
//
// This is the paper's other headline kernel (the matrix multiplication of Sections 3.1 and 5.2) on
// the same machinery as the attention kernel: both operand tiles travel global -> LDS with
// direct-to-LDS loads through a ring of STAGES stages (the aref ring of Section 3.3 with depth 4;
// s_waitcnt vmcnt plus one s_barrier per K tile stand in for the full/empty credits), and the
// 32x32x16 MFMA consumes them.  There is no producer wave: every wave issues its share of the copies
// three K tiles ahead and computes.
//
// Workgroup: 8 waves (two per SIMD) on a 256 x 256 tile of C; a wave owns 128 (m) x 64 (n) of it,
// i.e. 8 accumulator blocks.  The product is computed transposed, D = B_tile A_tile^T, so that a
// lane ends up with one row m of C and runs of four consecutive n: the 16-bit results leave as 8-byte
// stores (computed the other way round a lane would hold single elements of 16 different rows).
//
// Schedule of one wave, K tile j (32 wide, two MFMA k-steps):
//   wait for its own copies of stage j+1; barrier (everyone's stage j+1 is complete, nobody reads
//   stage j-1 any more); issue the copies of stage j+3 into the slot of j-1;
//   request the k-step-1 fragments of tile j; 8 MFMAs on the k-step-0 fragments, which were
//   requested during tile j-1 (stage j was already complete then) -- so the matrix core has work
//   the moment the barrier opens; request the k-step-0 fragments of tile j+1; 8 MFMAs on k-step 1.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gemm_launch.h"
#include "gfx950_prims.h"
#include "tile_schedule.h"

namespace {

constexpr int G_NW = 8;                 // waves per workgroup
constexpr int G_BM = 256, G_BN = 256;   // tile of C per workgroup
constexpr int G_BK = 32;                // K tile
constexpr int G_STAGES = 4;
constexpr int G_OPER_BYTES = G_BM * G_BK * 2;        // one operand tile in the LDS (16 KiB)
constexpr int G_STAGE_BYTES = 2 * G_OPER_BYTES;      // A tile, then B tile
constexpr int G_PIECES = G_OPER_BYTES / 1024;        // 1 KiB wave-transfers per operand tile (16 rows x 64 B each)
constexpr int G_PPW = G_PIECES / G_NW;               // ... per wave and operand
constexpr int G_LPG = 2 * G_PPW;                     // copies a wave issues per stage
constexpr int G_GROUP_M = 8;                         // tile rows per raster group (see tile_coords)
static_assert(G_BM == G_BN && G_PIECES % G_NW == 0, "operand tiles are copied the same way");

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

template <int DTYPE>
__global__ __launch_bounds__(G_NW * 64)
void gemm_nt_kernel(const uint16_t* __restrict__ A, const uint16_t* __restrict__ B, uint16_t* __restrict__ C,
                    int M, int N, int K, int ntm, int ntn)
{
    typedef Elem<DTYPE> E;
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const unsigned lds_base = (unsigned)(size_t)(LDS_AS void*)smem;

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int lr = lane & 31, g = lane >> 5;
    const int wm = wave & 1, wn = wave >> 1;                 // the wave's 128 x 64 block inside the tile

    int tm, tn;
    tile_coords(__builtin_amdgcn_readfirstlane(tile_schedule(ntm * ntn, (int)gridDim.x, (int)blockIdx.x, 0)), ntm, ntn, tm, tn);
    const int m0 = tm * G_BM, n0 = tn * G_BN;
    const int nk = K / G_BK;
    const size_t row_bytes = (size_t)K * 2;

    // ---- global -> LDS copies.  Operand tile in the LDS: [16-row block][16-byte column (4)][row (16)][16 B];
    // one copy instruction moves a 16-row block: lane L fetches row L%16, column L/16 (LDS offset 16*L).
    // Inside the matrix the per-lane offset is a constant and the piece / K-tile offset sits in the scalar
    // base; tiles that overhang the matrix clamp their rows (the surplus rows are never stored).
    const bool interior = m0 + G_BM <= M && n0 + G_BN <= N;
    const unsigned lane_off = (unsigned)((lane & 15) * row_bytes) + (lane >> 4) * 16;
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
            a_voff[i] = (unsigned)((size_t)min(m0 + p * 16 + (lane & 15), M - 1) * row_bytes) + (lane >> 4) * 16;
            b_voff[i] = (unsigned)((size_t)min(n0 + p * 16 + (lane & 15), N - 1) * row_bytes) + (lane >> 4) * 16;
        }
    }
    auto issue_stage = [&](int s) __attribute__((always_inline)) {
        const unsigned sbase = lds_base + (s % G_STAGES) * G_STAGE_BYTES + wave * (G_PPW * 1024);
        const size_t koff = (size_t)s * (G_BK * 2);
#pragma unroll
        for (int i = 0; i < G_PPW; ++i) dma16(a_piece[i] + koff, a_voff[i], sbase + i * 1024);
#pragma unroll
        for (int i = 0; i < G_PPW; ++i) dma16(b_piece[i] + koff, b_voff[i], sbase + G_OPER_BYTES + i * 1024);
    };

    // ---- fragments: 32 rows x 16 k of an operand tile; lane l holds row l%32, k = 16*ks + 8*(l/32) .. +7
    const int frag_lane = (lr >> 4) * 1024 + g * 256 + (lr & 15) * 16;
    struct Frags { s16x8 bn[2]; s16x8 am[4]; };        // B-matrix rows (n) feed the MFMA's A operand, A-matrix rows (m) its B operand
    auto read_frags = [&](int s, int ks) __attribute__((always_inline)) -> Frags {
        const char* st = smem + (s % G_STAGES) * G_STAGE_BYTES + frag_lane + ks * 512;
        Frags f;
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
            f.bn[nb] = *reinterpret_cast<const s16x8*>(st + G_OPER_BYTES + (wn * 2 + nb) * 2048);
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
            f.am[mb] = *reinterpret_cast<const s16x8*>(st + (wm * 4 + mb) * 2048);
        return f;
    };

    f32x16 acc[2][4];
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int mb = 0; mb < 4; ++mb) acc[nb][mb] = f32x16(0.f);
    auto mfmas = [&](const Frags& f) __attribute__((always_inline)) {
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) acc[nb][mb] = E::mfma(f.bn[nb], f.am[mb], acc[nb][mb]);
    };

    // ---- prologue: three stages in flight; stage 0 complete for everyone; first fragments requested
    issue_stage(0);
    if (nk > 1) issue_stage(1);
    if (nk > 2) issue_stage(2);
    if (nk > 2) wait_vmcnt<2 * G_LPG>(); else if (nk > 1) wait_vmcnt<G_LPG>(); else wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
    Frags f0 = read_frags(0, 0);
    __builtin_amdgcn_s_waitcnt(0xC07F);       // lgkmcnt(0): same state on both ways into the loop (see its end)

    // (bottom-tested: with the exit test at the top the accumulators would be copied every iteration)
    int j = 0;
    do {
        if (j + 2 < nk) wait_vmcnt<G_LPG>(); else wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();
        if (j + 3 < nk) issue_stage(j + 3);
        const Frags f1 = read_frags(j, 1);
        __builtin_amdgcn_sched_barrier(0);
        mfmas(f0);
        __builtin_amdgcn_sched_barrier(0);
        if (j + 1 < nk) f0 = read_frags(j + 1, 0);
        __builtin_amdgcn_sched_barrier(0);
        mfmas(f1);
        __builtin_amdgcn_sched_barrier(0);
        // The next tile's first fragments have landed long ago; saying so here keeps the compiler from
        // waiting for ALL outstanding LDS reads (the fresh k-step-1 requests included) at the loop top.
        __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0)
    } while (++j < nk);

    // ---- epilogue: lane holds row m of C and, per accumulator register quad, four consecutive n
    const bool vec_ok = (N & 3) == 0 && (reinterpret_cast<uintptr_t>(C) & 7) == 0;
#pragma unroll
    for (int mb = 0; mb < 4; ++mb) {
        const int m = m0 + wm * 128 + mb * 32 + lr;
        if (m >= M) continue;
        uint16_t* crow = C + (size_t)m * N;
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                const int n = n0 + wn * 64 + nb * 32 + i4 * 8 + g * 4;
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

template <int DTYPE>
int launch(const GemmLaunchArgs& a)
{
    constexpr int smem = G_STAGES * G_STAGE_BYTES;
    auto kern = gemm_nt_kernel<DTYPE>;
    static bool attr_set = false;   // idempotent; a race only repeats the call
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, smem) != hipSuccess)
            return -1;
        attr_set = true;
    }
    const uint16_t* A = (const uint16_t*)a.a;
    const uint16_t* B = (const uint16_t*)a.b;
    uint16_t* C = (uint16_t*)a.c;
    int M = a.M, N = a.N, K = a.K;
    int ntm = (M + G_BM - 1) / G_BM, ntn = (N + G_BN - 1) / G_BN;
    void* args[] = {&A, &B, &C, &M, &N, &K, &ntm, &ntn};
    const hipError_t e = hipLaunchKernel(reinterpret_cast<const void*>(kern), dim3((unsigned)(ntm * ntn)), dim3(G_NW * 64),
                                         args, smem, (hipStream_t)a.stream);
    return e == hipSuccess ? 0 : -1;
}

}  // namespace

int gemm_launch(const GemmLaunchArgs& a) { return a.dtype == 0 ? launch<0>(a) : launch<1>(a); }

int gemm_launch_tile_param(int which)
{
    switch (which) {
        case 0: return G_BM;
        case 1: return G_BN;
        case 2: return G_BK;
        case 3: return G_STAGES;
        case 4: return G_NW * 64;
        default: return -1;
    }
}
