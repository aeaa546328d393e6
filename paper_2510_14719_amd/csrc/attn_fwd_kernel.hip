// Fused attention forward for gfx950 (MI355X): O = softmax(scale * Q K^T [+ causal mask]) V and
// per-row log-sum-exp, in one kernel with a streaming softmax.
//
// The three stages of one key/value tile follow the paper's Section 3.4.2: T = Q K^T on the matrix
// cores, C = softmax on the vector ALU, U = P V on the matrix cores, and the goal is the one of its
// coarse-grained pipeline (Algorithm 1): keep the matrix cores busy while the vector ALU works.
//
// What carries over from the paper's Hopper design and what does not:
//  * Producer/consumer warp roles are gone.  Every wave issues its share of the global -> LDS copies
//    (direct-to-LDS loads, no register staging) two tiles ahead of their use.  The LDS holds a ring of
//    STAGES tiles, the counterpart of an aref ring of depth D (Section 3.3.2); one s_waitcnt plus one
//    s_barrier per tile play the role of the full/empty credits: a stage is overwritten only after
//    every wave has passed the barrier that follows its last read of it.
//  * A gfx950 wave issues in order and cannot run its own vector instructions under its own MFMA
//    (measured: one wave alternating 1 MFMA + n FMAs takes 41 + 4n cycles per pair), so the overlap of
//    Algorithm 1 cannot live inside one instruction stream.  It is realised BETWEEN the two waves that
//    share a SIMD: the eight waves of a workgroup form two groups of four (one wave of each group per
//    SIMD) that run the same pipeline half a period apart,
//        group A after barrier j:  [U_{j-1}, T_j] on the matrix cores, then C_j on the vector ALU
//        group B after barrier j:  C_j on the vector ALU, then [U_j, T_{j+1}] on the matrix cores
//    so while one wave of a SIMD streams 32 MFMAs the other one does its softmax.  The workgroup
//    barrier re-locks the two groups into opposite phases every tile.
//
// Register layout.  The scores are computed transposed, S^T = K Q^T, with the 32x32x16 MFMA: the
// K tile is the A operand (32 keys x 16 features), Q^T the B operand.  A lane then owns ONE query
// (column lane%32 of the result) and 16 of the 32 keys of a block; the other 16 keys of that query
// sit in lane^32.  Row maximum and row sum are in-lane operations plus one lane<->lane+32
// exchange, and the probabilities are already laid out as the B operand of the second contraction
// O^T = V^T P^T.  V^T fragments come from the LDS through the transposing 64-bit read of gfx950.

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "attn_launch.h"
#include "gfx950_prims.h"
#include "launch_once.h"
#include "tile_schedule.h"

namespace {

// The softmax reference moves only when a row maximum grew by more than this many powers of two.
constexpr float RESCALE_LOG2 = 8.0f;

// LDS fragments requested ahead of their MFMA inside a burst (see mfma_burst).
#ifndef ATTN_FWIN
#define ATTN_FWIN 2
#endif

// Independent accumulation chains of the row sum (see softmax_tile).
#ifndef ATTN_SUMCHAINS
#define ATTN_SUMCHAINS 4
#endif

// 1: launch one workgroup per resident slot and let each walk several tiles; 0: one workgroup per tile.
#ifndef ATTN_PERSISTENT
#define ATTN_PERSISTENT 1
#endif
// Longest sequence for which the non-causal d = 128 launch is persistent too (see launch_d).
#ifndef ATTN_PERSIST_NC_MAX_N
#define ATTN_PERSIST_NC_MAX_N 1024
#endif

// 1: the causal d = 64 launch is persistent as well (measured on MI355X: see launch_d).
#ifndef ATTN_PERSISTENT_D64
#define ATTN_PERSISTENT_D64 1
#endif

// 1: the d = 64 kernels are compiled for two resident workgroups per CU (128 registers per lane).  The one-tile-per-
// workgroup kernels need 113 registers and are resident in pairs anyway; the persistent causal one needs 168 (the next
// tile's Q fragments are loaded under the epilogue), and forced down to 128 it spills and gains nothing (measured on
// MI355X, c2 causal: 552 vs 548-558 TFLOP/s), so the knob is off.
#ifndef ATTN_D64_TWO_WG
#define ATTN_D64_TWO_WG 0
#endif

// Which wave group issues the global -> LDS copies (see COPY_WAVES in the kernel).
#ifndef ATTN_COPY_GROUP
#define ATTN_COPY_GROUP 0
#endif

// 1: in the steady state a wave issues its copies of a stage one at a time between the exponentials of the
// softmax; 0: as one block before the softmax (a wave is held ~270 cycles per tile by that block).  Measured
// on MI355X: spreading them loses 1-2 % (c3, c4, c5), and so does issuing the block at a different point
// of the softmax in each wave of a group: the ~70 cycles per copy instruction are not a queue, so the block stays.
#ifndef ATTN_COPIES_IN_SOFTMAX
#define ATTN_COPIES_IN_SOFTMAX 0
#endif

#ifdef ATTN_TIMING
// Profiling builds only: per-wave cycle totals of the main-loop sections of the first workgroups.
constexpr int DBG_WGS = 1024, DBG_SLOTS = ATTN_TIMING >= 3 ? 32 : 8;
__device__ unsigned long long attn_dbg[DBG_WGS * 8 * DBG_SLOTS];
#if ATTN_TIMING >= 2
#define TSTAMP(var) unsigned long long var; __builtin_amdgcn_sched_barrier(0); \
    asm volatile("s_memtime %0\n\ts_waitcnt lgkmcnt(0)" : "=s"(var) :: "memory"); __builtin_amdgcn_sched_barrier(0)
#if ATTN_TIMING >= 3   // absolute stamps of iterations 100..103
#define TACC(slot, a, b) if (j >= 100 && j < 104) { dbg_acc[8 + (j - 100) * 5 + slot] = (a); if (slot == 3) dbg_acc[8 + (j - 100) * 5 + 4] = (b); }
#else
#define TACC(slot, a, b) dbg_acc[slot] += (b) - (a)
#endif
#else
#define TSTAMP(var)
#define TACC(slot, a, b)
#endif
#else
#define TSTAMP(var)
#define TACC(slot, a, b)
#endif

// Exchange with lane^32 (v_permlane32_swap swaps the upper 32 lanes of its first operand with the
// lower 32 lanes of its second): afterwards `a` holds the lower half's values on every lane and `b`
// the upper half's, so op(a, b) is the two-lane reduction on all 64 lanes.  Written as inline asm
// because clang 22 folds the two results of __builtin_amdgcn_permlane32_swap into one
// (fmax(r[0], r[1]) is compiled as r[0]), which silently drops the partner lane.  The s_nop covers
// the VALU-write -> permlane-read hazard the compiler would otherwise handle.
__device__ __forceinline__ void swap32(float& a, float& b) {
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
}
__device__ __forceinline__ float xor32_max(float x) {
    float a = x, b = x;
    swap32(a, b);
    return __builtin_fmaxf(a, b);
}
__device__ __forceinline__ float xor32_sum(float x) {
    float a = x, b = x;
    swap32(a, b);
    return a + b;
}

// (d = 64: the LDS ring is 64 KiB, two workgroups fit a CU; the second launch bound, waves per SIMD, asks the
// compiler for the 128 registers per lane that let their 16 waves be resident together)
template <int DTYPE, int D, int NW, int MB, int BN, int STAGES, bool CAUSAL, bool PERSIST>
__global__ __launch_bounds__(NW * 64, (D == 64 && ATTN_D64_TWO_WG) ? 4 : 1)
void attn_fwd_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
                     uint16_t* __restrict__ o, float* __restrict__ lse, int N, int nqt, int total,
                     float scale, float scale_log2e)
{
    typedef Elem<DTYPE> E;
    constexpr int BM = NW * MB * 32;            // query rows per workgroup
    constexpr int KB = BN / 32;                 // 32-key blocks per K/V tile
    constexpr int KK = D / 16;                  // contraction steps of Q K^T
    constexpr int DB = D / 32;                  // 32-wide feature blocks of O
    constexpr int ROW_BYTES = D * 2;
    constexpr int TILE_BYTES = BN * ROW_BYTES;  // one K or one V tile
    constexpr int STAGE_BYTES = 2 * TILE_BYTES;
    constexpr int RB = BN / 16;                 // 16-row blocks per tile
    constexpr int CHUNKS = TILE_BYTES / 1024;   // 1 KiB wave-transfers per tile
    // Which waves issue the copies: 0 = all eight, 1 = group B only, 2 = group A only.
    constexpr int NG = NW / 4;                  // wave groups: one wave of each group per SIMD
    constexpr int COPY_WAVES = NG == 3 ? 8 : (ATTN_COPY_GROUP == 0 ? NW : NW / 2);
    constexpr int CPW = CHUNKS / COPY_WAVES;    // ... per copying wave
    constexpr int LPG = 2 * CPW;                // copies such a wave issues per stage (K part + V part)
    static_assert(CHUNKS % COPY_WAVES == 0, "tile must split evenly over the copying waves");
    static_assert(STAGES == 4, "the ring protocol below keeps four stages");
    static_assert(NW == 8 || NW == 12, "two or three groups of four waves, one wave of each group per SIMD");

#ifdef ATTN_TIMING
    const unsigned long long rt_kernel_entry = __builtin_amdgcn_s_memrealtime();
#endif
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const unsigned lds_base = (unsigned)(size_t)(LDS_AS void*)smem;

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform, kept in an SGPR
    const int lane = threadIdx.x & 63;
    const int lr = lane & 31, g = lane >> 5;
    const int group = __builtin_amdgcn_readfirstlane(wave >> 2);   // waves w, w + 4 (, w + 8) share a SIMD
    const bool group_b = group == NG - 1;       // the group that does its softmax first

    // ---- which (batch*head, query tile) the workgroup works on: set per round of the tile schedule
    int round = 0;
    int logical __attribute__((unused)), bh, wq0, nt, nt_w;             // nt: K/V tiles the workgroup walks; nt_w: those this wave computes on
    size_t head_off;
    const uint16_t* qh;
    const char *kh, *vh;
    auto set_tile = [&](int tile) __attribute__((always_inline)) {
        tile = __builtin_amdgcn_readfirstlane(tile);   // wave-uniform by construction; keeps all of the below in SGPRs
        logical = tile;
        bh = __builtin_amdgcn_readfirstlane(tile / nqt);   // (the division runs on the vector ALU)
        int qt = tile - bh * nqt;
        if (CAUSAL) qt = nqt - 1 - qt;          // long rows first
        const int q0 = qt * BM;
        wq0 = q0 + wave * (MB * 32);            // first query row of this wave
        head_off = (size_t)bh * N * D;
        qh = q + head_off;
        kh = reinterpret_cast<const char*>(k + head_off);
        vh = reinterpret_cast<const char*>(v + head_off);
        nt = (N + BN - 1) / BN;
        if (CAUSAL) {
            const int last_q = min(q0 + BM, N) - 1;
            nt = min(nt, last_q / BN + 1);
        }
        nt_w = nt;
        if (CAUSAL) nt_w = min(nt, (wq0 + MB * 32 - 1) / BN + 1);   // later tiles are wholly hidden from this wave's rows
        // All of these are wave-uniform; say so, or values that cross the tile loop end up in vector registers.
        nt = __builtin_amdgcn_readfirstlane(nt);
        nt_w = __builtin_amdgcn_readfirstlane(nt_w);
        wq0 = __builtin_amdgcn_readfirstlane(wq0);
        kh = uniform_ptr(kh);
        vh = uniform_ptr(vh);
    };
    set_tile(tile_schedule(total, (int)gridDim.x, (int)blockIdx.x, 0));   // the launcher keeps grid <= total

    // ---- global -> LDS copies.  Stage s of the ring holds K tile s+1 and V tile s: the pair that one
    // MFMA burst reads (U_s needs V_s, T_{s+1} needs K_{s+1}).  A wave moves CPW 1 KiB pieces of each.
    // K tile in LDS: [feature group of 32][16-row block][16-byte column of the group (4)][row (16)][16 B]
    // V tile in LDS: [feature group of 32][row (BN)][64 B]
    // Lane L of a K piece fetches row L%16, column L/16 of the piece's (16 rows x 64 B) source block; of
    // a V piece row L/4, column L%4.  Inside the sequence the per-lane offset is a constant and the
    // tile/piece offset is added to the scalar base; the clamped form serves tiles that overrun the
    // sequence (their surplus rows are masked or never read).
    const unsigned k_lane_off = (lane & 15) * ROW_BYTES + (lane >> 4) * 16;
    const unsigned v_lane_off = (lane >> 2) * ROW_BYTES + (lane & 3) * 16;
    // does this wave issue copies, and its index among the copying waves (three groups: the first eight waves)
    const bool copies = NG == 3 ? wave < 8 : (ATTN_COPY_GROUP == 0 || (ATTN_COPY_GROUP == 1) == group_b);
    const int cwave = (NG == 3 || ATTN_COPY_GROUP == 0) ? wave : (wave & (NW / 2 - 1));
    int piece_src[CPW], piece_dst[CPW];         // wave-uniform: source offset inside a tile, LDS offset inside a K or V slot
#pragma unroll
    for (int i = 0; i < CPW; ++i) {
        const int wc = cwave * CPW + i, fg = wc / RB, rb = wc % RB;
        piece_src[i] = rb * 16 * ROW_BYTES + fg * 64;
        piece_dst[i] = wc * 1024;
    }
    auto issue_stage = [&](int s) __attribute__((always_inline)) {             // s = -1 is the stage that only brings K tile 0
        if (!copies) return;
        const unsigned sbase = lds_base + ((s + STAGES) % STAGES) * STAGE_BYTES;
        if (s >= 0 && (s + 2) * BN <= N) {      // K tile s+1 and V tile s lie wholly inside the sequence
            const char* kt = kh + (size_t)(s + 1) * TILE_BYTES;
            const char* vt = vh + (size_t)s * TILE_BYTES;
#pragma unroll
            for (int i = 0; i < CPW; ++i) dma16(kt + piece_src[i], k_lane_off, sbase + piece_dst[i]);
#pragma unroll
            for (int i = 0; i < CPW; ++i) dma16(vt + piece_src[i], v_lane_off, sbase + TILE_BYTES + piece_dst[i]);
        } else {
#pragma unroll
            for (int i = 0; i < CPW; ++i) {
                const int wc = cwave * CPW + i, fg = wc / RB, rb = wc % RB;
                const int row = min(max((s + 1) * BN + rb * 16 + (lane & 15), 0), N - 1);
                dma16(kh, (unsigned)(row * ROW_BYTES + fg * 64 + (lane >> 4) * 16), sbase + piece_dst[i]);
            }
#pragma unroll
            for (int i = 0; i < CPW; ++i) {
                const int wc = cwave * CPW + i, fg = wc / RB, rb = wc % RB;
                const int row = min(max(s * BN + rb * 16 + (lane >> 2), 0), N - 1);
                dma16(vh, (unsigned)(row * ROW_BYTES + fg * 64 + (lane & 3) * 16), sbase + TILE_BYTES + piece_dst[i]);
            }
        }
    };

    // One copy of a stage that lies wholly inside the sequence: K piece i < CPW, else V piece i - CPW.
    auto issue_piece_inside = [&](int s, int i) __attribute__((always_inline)) {
        const unsigned sbase = lds_base + ((s + STAGES) % STAGES) * STAGE_BYTES;
        if (i < CPW) dma16(kh + (size_t)(s + 1) * TILE_BYTES + piece_src[i], k_lane_off, sbase + piece_dst[i]);
        else dma16(vh + (size_t)s * TILE_BYTES + piece_src[i - CPW], v_lane_off, sbase + TILE_BYTES + piece_dst[i - CPW]);
    };

    // ---- prologue of a tile: three stages in flight, Q fragments into registers
    s16x8 Qf[MB][KK];
    auto prologue = [&]() __attribute__((always_inline)) {
        issue_stage(-1);
        issue_stage(0);
        issue_stage(1);
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            const int row = min(wq0 + mb * 32 + lr, N - 1);
            const uint16_t* qr = qh + (size_t)row * D;
#pragma unroll
            for (int kk = 0; kk < KK; ++kk)
                Qf[mb][kk] = *reinterpret_cast<const s16x8*>(qr + (kk * 2 + g) * 8);
        }
    };
    prologue();

    f32x16 O[MB][DB], S[MB][KB];
    unsigned pw[MB][KB * 8];                    // P of the current tile as packed 16-bit pairs
    float m_run[MB], l_run[MB];

    // per-lane LDS read offsets (the rest of every address is an immediate)
    const int k_lane = (lr >> 4) * 1024 + g * 256 + (lr & 15) * 16;
    const int v_lane = TILE_BYTES + (4 * g + ((lane & 15) >> 2)) * 64 + ((lane >> 4) & 1) * 32 + (lane & 3) * 8;

    // K fragment (A operand of T): keys kb*32 + lane%32, features (kk*2 + lane/32)*8 .. +7
    auto read_kf = [&](const char* sk, int kb, int kk) __attribute__((always_inline)) -> s16x8 {
        return *reinterpret_cast<const s16x8*>(sk + ((kk >> 1) * RB + kb * 2) * 1024 + (kk & 1) * 512);
    };
    // V^T fragment (A operand of U): features db*32 + lane%32, the 8 keys of block kb that the P
    // operand of MFMA ks holds in this lane group, fetched with the transposing LDS read
    auto read_vf = [&](const char* sv, int kb, int ks, int db) __attribute__((always_inline)) -> s16x8 {
        const char* a = sv + db * (BN * 64) + (kb * 32 + ks * 16) * 64;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(a));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(a + 8 * 64));
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    };

    // ---- MFMA burst on one stage: U (O^T += V^T P^T with the P in pw) and/or T (S^T = K Q^T), as one
    // stream of MFMAs whose LDS fragments are requested FWIN MFMAs ahead.  The scheduling barriers
    // keep that order: left alone the compiler requests each fragment right before its MFMA.
    auto mfma_burst = [&](auto do_u, auto do_t, const char* stage_ptr) __attribute__((always_inline)) {
        constexpr int NU = decltype(do_u)::value ? KB * 2 * DB : 0;
        constexpr int NT = decltype(do_t)::value ? KB * KK : 0;
        constexpr int NF = NU + NT;
        constexpr int FWIN = ATTN_FWIN < NF ? ATTN_FWIN : NF;
        const char* sk = stage_ptr + k_lane;
        const char* sv = stage_ptr + v_lane;
        s16x8 fr[NF];
        auto fetch = [&](int f) __attribute__((always_inline)) {
            if (f < NU) fr[f] = read_vf(sv, f / (2 * DB), (f / DB) % 2, f % DB);
            else fr[f] = read_kf(sk, (f - NU) % KB, (f - NU) / KB);
        };
        auto run_mfma = [&](int f) __attribute__((always_inline)) {
            if (f < NU) {
                const int kb = f / (2 * DB), ks = (f / DB) % 2, db = f % DB;
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    u32x4 w;
#pragma unroll
                    for (int t = 0; t < 4; ++t) w[t] = pw[mb][kb * 8 + ks * 4 + t];
                    O[mb][db] = E::mfma(fr[f], __builtin_bit_cast(s16x8, w), O[mb][db]);
                }
            } else {
                const int kb = (f - NU) % KB, kk = (f - NU) / KB;
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    S[mb][kb] = E::mfma(fr[f], Qf[mb][kk], kk == 0 ? f32x16(0.f) : S[mb][kb]);
                }
            }
        };
#pragma unroll
        for (int f = 0; f < FWIN; ++f) fetch(f);
#pragma unroll
        for (int f = 0; f < NF; ++f) {
            if (f + FWIN < NF) fetch(f + FWIN);
            run_mfma(f);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // ---- C of tile j: mask, streaming softmax of S into pw, running maximum / sum, rescaling of O.
    // Base-2 exponentials with the scale folded into the exponent.  The running reference m only
    // moves when a row maximum grew by more than 2^RESCALE_LOG2 (the probabilities then stay below
    // that factor), so the rescaling of O is rare after the first tiles.
    // With `spread` the wave's copies of stage j + 2 (known to lie inside the sequence) go out between the
    // exponentials, evenly spaced.
    // `part`: 0 = the whole tile; 1 = mask, maximum, reference, rescaling and the first half of the score pairs;
    // 2 = the second half of the pairs and the row sum (the middle group of three splits its softmax around its burst).
    float part_negmc[MB], part_sum[MB][ATTN_SUMCHAINS];
    auto softmax_tile = [&](int j, auto spread, auto part) __attribute__((always_inline)) {
        constexpr bool SPREAD = decltype(spread)::value;
        constexpr int PART = decltype(part)::value;
        constexpr int NPAIR = KB * 8, NCOPY = 2 * CPW, PER = NPAIR / NCOPY;
        static_assert(!SPREAD || (PER >= 1 && PER * NCOPY == NPAIR), "copies spread evenly over the exponentials");
        const int kv0 = j * BN;
        if (PART != 2 && ((kv0 + BN > N) || (CAUSAL && kv0 + BN - 1 > wq0))) {
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                const int qi = wq0 + mb * 32 + lr;
                const int lim = CAUSAL ? min(qi, N - 1) : N - 1;   // last visible key
#pragma unroll
                for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int key = kv0 + kb * 32 + (i >> 2) * 8 + g * 4 + (i & 3);
                        if (key > lim) S[mb][kb][i] = -__builtin_inff();
                    }
            }
        }
        float alpha[MB];
        bool upd_any = false;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            // independent chains: a dot2 accumulate has a dependent latency of about four issue slots
            constexpr int NCH = ATTN_SUMCHAINS;
            float sum[NCH];
            float neg_mc;
            alpha[mb] = 1.0f;
            if (PART != 2) {
                float mx = S[mb][0][0];
#pragma unroll
                for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) mx = __builtin_fmaxf(mx, S[mb][kb][i]);
                mx = xor32_max(mx);
                const float m_old = m_run[mb];
                const float m_new = __builtin_fmaxf(m_old, mx);
                const bool upd = (m_new - m_old) * scale_log2e > RESCALE_LOG2;
                const float m_use = upd ? m_new : m_old;
                upd_any |= upd;
                alpha[mb] = __builtin_amdgcn_exp2f((m_old - m_use) * scale_log2e);
                neg_mc = -m_use * scale_log2e;
                m_run[mb] = m_use;
#pragma unroll
                for (int c = 0; c < NCH; ++c) sum[c] = 0.f;
            } else {
                neg_mc = part_negmc[mb];
#pragma unroll
                for (int c = 0; c < NCH; ++c) sum[c] = part_sum[mb][c];
            }
#pragma unroll
            for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                for (int t = 0; t < 8; ++t) {
                    if ((PART == 1 && kb * 8 + t >= NPAIR / 2) || (PART == 2 && kb * 8 + t < NPAIR / 2)) continue;
                    const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(S[mb][kb][2 * t], scale_log2e, neg_mc));
                    const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(S[mb][kb][2 * t + 1], scale_log2e, neg_mc));
                    const unsigned w = E::pack2(p0, p1);
                    pw[mb][kb * 8 + t] = w;
                    sum[t % NCH] = E::add_pair(w, sum[t % NCH]);
                    if (SPREAD && mb == 0 && (kb * 8 + t) % PER == PER / 2) {
                        __builtin_amdgcn_sched_barrier(0);
                        if (copies) issue_piece_inside(j + 2, (kb * 8 + t) / PER);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            if (PART == 1) {                    // the second half continues these sums with this reference
                part_negmc[mb] = neg_mc;
#pragma unroll
                for (int c = 0; c < NCH; ++c) part_sum[mb][c] = sum[c];
                l_run[mb] = l_run[mb] * alpha[mb];
            } else {
                float tile_sum = sum[0];
#pragma unroll
                for (int c = 1; c < NCH; ++c) tile_sum += sum[c];
                l_run[mb] = l_run[mb] * alpha[mb] + tile_sum;
            }
        }
        if (PART != 2 && __builtin_amdgcn_ballot_w64(upd_any) != 0) {
            // whole-vector multiplies: element-wise updates would make the compiler split the
            // accumulator tuples into scalars and re-assemble them around every MFMA
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int db = 0; db < DB; ++db) O[mb][db] = O[mb][db] * alpha[mb];
        }
    };

    // At barrier j every wave's share of stages <= j has landed (each wave waits for its own copies up
    // to stage j, leaving only stage j+1's in flight) and nobody reads stage j-2 any more, so that
    // stage takes the copies of stage j+2.
    auto wait_stage = [&](int j) __attribute__((always_inline)) {
        if (copies) {
            if (j + 1 < nt) wait_vmcnt<LPG>(); else wait_vmcnt<0>();
        }
        __builtin_amdgcn_s_barrier();
    };
    auto stage_ptr = [&](int s) __attribute__((always_inline)) -> const char* { return smem + ((s + STAGES) % STAGES) * STAGE_BYTES; };

    // ---- epilogue: normalise, write O (16-bit) and LSE (natural log).  Expanded at the end of each
    // group's code path, so that the accumulators of the two paths never have to meet in one register set.
    auto epilogue = [&](size_t ep_head_off, int ep_bh, int ep_wq0) __attribute__((always_inline)) {
    uint16_t* oh = o + ep_head_off;
    float* lh = lse + (size_t)ep_bh * N;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const float l_tot = xor32_sum(l_run[mb]);
        const float inv = 1.0f / l_tot;
        const int row = ep_wq0 + mb * 32 + lr;
        if (row < N) {
            if (g == 0) lh[row] = m_run[mb] * scale + __builtin_logf(l_tot);
            uint16_t* orow = oh + (size_t)row * D;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) {
                    u32x2 w;
                    w[0] = E::pack2(O[mb][db][i4 * 4 + 0] * inv, O[mb][db][i4 * 4 + 1] * inv);
                    w[1] = E::pack2(O[mb][db][i4 * 4 + 2] * inv, O[mb][db][i4 * 4 + 3] * inv);
                    *reinterpret_cast<u32x2*>(orow + db * 32 + i4 * 8 + g * 4) = w;
                }
        }
    }
    };

    // ---- end of a tile: when the schedule has another tile for this workgroup, its prologue is issued
    // first (after a barrier: every wave is then done reading the ring), so that its copies and Q
    // loads are in flight while the epilogue of the finished tile normalises and stores.
    bool more = true;
    auto finish_tile = [&]() __attribute__((always_inline)) {
        const size_t ep_head_off = head_off;
        const int ep_bh = bh, ep_wq0 = wq0;
        const int next = PERSIST ? tile_schedule(total, (int)gridDim.x, (int)blockIdx.x, ++round) : -1;
        more = next >= 0;
        if (more) {
            __builtin_amdgcn_s_barrier();
            set_tile(next);
            prologue();
        }
        epilogue(ep_head_off, ep_bh, ep_wq0);
    };

#ifdef ATTN_TIMING
    unsigned long long dbg_acc[DBG_SLOTS] = {};
    unsigned long long rt0 = 0, ct0 = 0;
#endif
    do {
    // (the tile's coordinates are derived afresh from the round number: only that number and the Q
    // fragments cross from one tile to the next, everything else restarts from scalar registers)
    set_tile(tile_schedule(total, (int)gridDim.x, (int)blockIdx.x, __builtin_amdgcn_readfirstlane(round)));
    // Use the Q fragments once here: the compiler then waits for their loads before the loop instead
    // of inside it, where its vmcnt(0) would also wait for the K/V copies issued a moment earlier.
    // (The Q loads were issued after the copies of the prologue, so this wait also covers stages -1, 0, 1.)
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) asm volatile("" :: "v"(Qf[mb][kk]));
    wait_vmcnt<0>();
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        m_run[mb] = -__builtin_inff();
        l_run[mb] = 0.f;
#pragma unroll
        for (int db = 0; db < DB; ++db) O[mb][db] = f32x16(0.f);
    }
    __builtin_amdgcn_s_barrier();               // stages -1, 0, 1 are complete for every wave
#ifdef ATTN_TIMING
    rt0 = __builtin_amdgcn_s_memrealtime(); ct0 = __builtin_readcyclecounter();
#endif
    // Each group's steady state is one loop with a single code path (the first and last tile and the
    // idle tail of a causal wave are peeled off), so the accumulators stay in place across iterations.
    constexpr std::integral_constant<int, 0> WHOLE{};
    constexpr std::integral_constant<int, 1> FIRST_HALF{};
    constexpr std::integral_constant<int, 2> SECOND_HALF{};
    if (NG == 3 && group == 1) {
        // the middle group of three, iteration j: second half of C_j, then [U_j, T_{j+1}], then the first half of
        // C_{j+1}; both contractions read stage j.  Its burst falls between those of the first group (right after
        // the barrier) and of the last (after its whole softmax): three bursts per SIMD and tile, back to back.
        mfma_burst(std::false_type{}, std::true_type{}, stage_ptr(-1));                  // T_0
        softmax_tile(0, std::false_type{}, FIRST_HALF);
        int j = 0;
        if (j + 1 < nt_w) {
            do {                                // bottom-tested: see group A
                wait_stage(j);
                if (j + 2 < nt) issue_stage(j + 2);
                softmax_tile(j, std::false_type{}, SECOND_HALF);
                mfma_burst(std::true_type{}, std::true_type{}, stage_ptr(j));
                softmax_tile(j + 1, std::false_type{}, FIRST_HALF);
            } while (++j + 1 < nt_w);
        }
        wait_stage(j);                                                                   // j == nt_w - 1
        if (j + 2 < nt) issue_stage(j + 2);
        softmax_tile(j, std::false_type{}, SECOND_HALF);
        mfma_burst(std::true_type{}, std::false_type{}, stage_ptr(j));                   // U of the last tile
        for (++j; j < nt; ++j) {                                                         // idle tail of a causal wave
            wait_stage(j);
            if (j + 2 < nt) issue_stage(j + 2);
        }
        finish_tile();
    } else if (!group_b) {
        // group A, iteration j: [U_{j-1}, T_j] then C_j; both contractions read stage j-1
        wait_stage(0);
        mfma_burst(std::false_type{}, std::true_type{}, stage_ptr(-1));                  // T_0
        if (2 < nt) issue_stage(2);
        softmax_tile(0, std::false_type{}, WHOLE);
        auto iter_a = [&](int j, auto spread) __attribute__((always_inline)) {
            TSTAMP(t0);
            wait_stage(j);
            TSTAMP(t1);
            mfma_burst(std::true_type{}, std::true_type{}, stage_ptr(j - 1));
            TSTAMP(t2);
            if (!decltype(spread)::value && j + 2 < nt) issue_stage(j + 2);
            TSTAMP(t3);
            softmax_tile(j, spread, WHOLE);
            TSTAMP(t4);
            TACC(0, t0, t1); TACC(1, t1, t2); TACC(2, t2, t3); TACC(3, t3, t4);
        };
        // (bottom-tested on purpose: with the exit test at the top the accumulators' loop-carried
        // value is also live on the exit edge, the first MFMA of an iteration then cannot update it
        // in place, and the compiler copies all 64 accumulator registers back every iteration)
        int j = 1;
        // iterations whose stage j + 2 exists and lies wholly inside the sequence spread its copies
        const int j_spread = ATTN_COPIES_IN_SOFTMAX ? min(nt_w, min(nt - 2, N / BN - 3)) : 0;
        if (j < j_spread) {
            do {
                iter_a(j, std::true_type{});
            } while (++j < j_spread);
        }
        if (j < nt_w) {
            do {
                iter_a(j, std::false_type{});
            } while (++j < nt_w);
        }
        if (j < nt) wait_stage(j);                                                       // j == nt_w
        mfma_burst(std::true_type{}, std::false_type{}, stage_ptr(j - 1));               // U of the last tile
        if (j < nt && j + 2 < nt) issue_stage(j + 2);
        for (++j; j < nt; ++j) {                                                         // idle tail of a causal wave
            wait_stage(j);
            if (j + 2 < nt) issue_stage(j + 2);
        }
        finish_tile();
    } else {
        // group B, iteration j: C_j then [U_j, T_{j+1}]; both contractions read stage j
        mfma_burst(std::false_type{}, std::true_type{}, stage_ptr(-1));                  // T_0
        auto iter_b = [&](int j, auto spread) __attribute__((always_inline)) {
            TSTAMP(t0);
            wait_stage(j);
            TSTAMP(t1);
            if (!decltype(spread)::value && j + 2 < nt) issue_stage(j + 2);
            TSTAMP(t2);
            softmax_tile(j, spread, WHOLE);
            TSTAMP(t3);
            mfma_burst(std::true_type{}, std::true_type{}, stage_ptr(j));
            TSTAMP(t4);
            TACC(0, t0, t1); TACC(2, t1, t2); TACC(3, t2, t3); TACC(1, t3, t4);
        };
        int j = 0;
        const int j_spread = ATTN_COPIES_IN_SOFTMAX ? min(nt_w - 1, min(nt - 2, N / BN - 3)) : 0;
        if (j < j_spread) {
            do {
                iter_b(j, std::true_type{});
            } while (++j < j_spread);
        }
        if (j + 1 < nt_w) {
            do {
                iter_b(j, std::false_type{});
            } while (++j + 1 < nt_w);
        }
        wait_stage(j);                                                                   // j == nt_w - 1
        if (j + 2 < nt) issue_stage(j + 2);
        softmax_tile(j, std::false_type{}, WHOLE);
        mfma_burst(std::true_type{}, std::false_type{}, stage_ptr(j));                   // U of the last tile
        for (++j; j < nt; ++j) {                                                         // idle tail of a causal wave
            wait_stage(j);
            if (j + 2 < nt) issue_stage(j + 2);
        }
        finish_tile();
    }
    } while (more);
#ifdef ATTN_TIMING
    if (blockIdx.x < DBG_WGS && lane == 0) {
        dbg_acc[5] = nt;
        dbg_acc[6] = __builtin_amdgcn_s_memrealtime() - rt0;   // 100 MHz ticks
        dbg_acc[7] = __builtin_readcyclecounter() - ct0;
#if ATTN_TIMING == 1
        dbg_acc[0] = rt0;                                        // absolute start of the main loop
        dbg_acc[1] = __builtin_amdgcn_s_getreg((31 << 11) | (0 << 6) | 4);    // HW_ID
        dbg_acc[2] = __builtin_amdgcn_s_getreg((31 << 11) | (0 << 6) | 20);   // XCC_ID
        dbg_acc[3] = logical;
        dbg_acc[4] = rt_kernel_entry;
#endif
        for (int i = 0; i < DBG_SLOTS; ++i) attn_dbg[(blockIdx.x * 8 + wave) * DBG_SLOTS + i] = dbg_acc[i];
    }
#endif

#ifdef ATTN_TIMING
    if (blockIdx.x < DBG_WGS && lane == 0) attn_dbg[(blockIdx.x * 8 + wave) * DBG_SLOTS + 5] = __builtin_amdgcn_s_memrealtime();
#endif
}

template <int DTYPE, int D, int NW, int MB, int BN, int STAGES, bool CAUSAL, bool PERSIST>
int launch(const AttnLaunchArgs& a)
{
    constexpr int BM = NW * MB * 32;
    constexpr int smem = STAGES * 2 * BN * D * 2;
    auto kern = attn_fwd_kernel<DTYPE, D, NW, MB, BN, STAGES, CAUSAL, PERSIST>;
    static PerDeviceOnce once;                  // the attribute belongs to the (kernel, device) pair
    const int dev = once.prepare(reinterpret_cast<const void*>(kern), smem);
    if (dev < 0) return -1;
    const int nqt = (a.N + BM - 1) / BM;
    const long long total = (long long)nqt * a.B * a.H;
    // Persistent launch: as many workgroups as the chip holds at once (one per CU at d = 128: the LDS
    // ring takes 128 KiB), each walking its share of the tile schedule.
    long long grid = total;
    if (PERSIST) {
        const int cus = once.compute_units(dev);
        if (cus < 8) return -1;
        const long long resident = (long long)cus * ((160 * 1024) / smem);
        if (grid > resident) grid = resident;
    }
    const float log2e = 1.4426950408889634f;
    const uint16_t* q = (const uint16_t*)a.q;
    const uint16_t* k = (const uint16_t*)a.k;
    const uint16_t* v = (const uint16_t*)a.v;
    uint16_t* o = (uint16_t*)a.o;
    float* lse = a.lse;
    int N = a.N, nqt_arg = nqt, total_arg = (int)total;
    float scale = a.scale, scale_log2e = a.scale * log2e;
    void* args[] = {&q, &k, &v, &o, &lse, &N, &nqt_arg, &total_arg, &scale, &scale_log2e};
    // the launch's own status, not hipGetLastError(): that one also reports stale errors of unrelated calls
    const hipError_t e = hipLaunchKernel(reinterpret_cast<const void*>(kern), dim3((unsigned)grid), dim3(NW * 64),
                                         args, smem, (hipStream_t)a.stream);
    return e == hipSuccess ? 0 : -1;
}

template <int DTYPE, int D>
int launch_d(const AttnLaunchArgs& a)
{
    constexpr int NW = D == 128 ? ATTN_CFG_NW : 8, MB = D == 64 ? ATTN_CFG_MB_D64 : ATTN_CFG_MB, BN = ATTN_CFG_BN, STAGES = ATTN_CFG_STAGES;
    // When the persistent form is used (d = 128 only: at d = 64 two workgroups share a CU and cover each
    // other's prologue and epilogue, and the next tile's Q fragments would cost the registers that let
    // them co-reside).  Causal: always; measured +2.5 % at N = 8192 (balanced tile lengths, next
    // prologue under the epilogue).  Without the mask all tiles are equally long and the hardware's own
    // dispatch balances as well; the persistent form only pays while a tile is short enough for its
    // prologue and epilogue to matter, and its main loop compiles slightly looser (-0.3 % at N = 16384).
    if (D == 128 && ATTN_PERSISTENT) {
        if (a.causal) return launch<DTYPE, D, NW, MB, BN, STAGES, true, true>(a);
        if (a.N <= ATTN_PERSIST_NC_MAX_N) return launch<DTYPE, D, NW, MB, BN, STAGES, false, true>(a);
    }
    if (D == 64 && ATTN_PERSISTENT_D64 && a.causal) return launch<DTYPE, D, NW, MB, BN, STAGES, true, true>(a);
    return a.causal ? launch<DTYPE, D, NW, MB, BN, STAGES, true, false>(a) : launch<DTYPE, D, NW, MB, BN, STAGES, false, false>(a);
}

}  // namespace

int attn_launch(const AttnLaunchArgs& a)
{
    if (ATTN_CFG_PIPE && a.d == 128) return attn_pipe_launch(a);
    if (a.dtype == 0) return a.d == 128 ? launch_d<0, 128>(a) : launch_d<0, 64>(a);
    return a.d == 128 ? launch_d<1, 128>(a) : launch_d<1, 64>(a);
}

#ifdef ATTN_TIMING
extern "C" int attn_dbg_read(unsigned long long* host, int n)
{
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(attn_dbg), sizeof(unsigned long long) * n);
}
#endif

int attn_launch_tile_param(int d, int causal, int which)
{
    (void)causal;
    if (d != 64 && d != 128) return -1;
    if (ATTN_CFG_PIPE && d == 128) {
        switch (which) {
            case 0: return 256;
            case 1: return 64;
            case 2: return 5;
            case 3: return ATTNP_CFG_NW * 64;
            default: return -1;
        }
    }
    switch (which) {
        case 0: return (d == 128 ? ATTN_CFG_NW : 8) * (d == 64 ? ATTN_CFG_MB_D64 : ATTN_CFG_MB) * 32;
        case 1: return ATTN_CFG_BN;
        case 2: return ATTN_CFG_STAGES;
        case 3: return (d == 128 ? ATTN_CFG_NW : 8) * 64;
        default: return -1;
    }
}
