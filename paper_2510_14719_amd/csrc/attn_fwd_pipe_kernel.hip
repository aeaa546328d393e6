// Fused attention forward for gfx950 (MI355X), 16-bit inputs, with the paper's coarse-grained
// pipeline (Section 3.4.2, Algorithm 1) INSIDE every wave's instruction stream.
//
// The three stages of a key/value tile are T = Q K^T (matrix cores), C = softmax (vector ALU) and
// U = P V (matrix cores).  A gfx950 wave issues in order, but an MFMA only occupies its wave for the
// issue slot: measured on the device, one wave alternating a 32-cycle MFMA with n independent
// vector instructions needs max(32, ~5 n) cycles per pair, not the sum.  So in iteration j a wave
// issues the MFMAs of T_{j+1} and U_{j-1} and, between them, the vector work of C_j in small
// slices: the matrix pipe runs back to back while the vector ALU works in its shadow, which is
// Algorithm 1 with "issue" and "commit" replaced by program order and the hardware's dependency
// checks.  S and P are double buffered in registers by tile parity, the loop is unrolled by two.
//
// Because one wave keeps its SIMD's matrix pipe busy on its own, a wave can own a whole SIMD and
// with it 512 registers: 64 query rows per wave (MB = 2) instead of 32.  Every K and V fragment read
// from the LDS then feeds two MFMAs (half the LDS traffic per flop), and consecutive MFMAs share
// one operand (less switching on the operand buses, which matters on a chip whose clock is set by
// its power limit).  The kernel is also instantiated with eight waves of 32 rows.
//
// Data movement is the ring of the paper's aref channel (Sections 3.2-3.3) without its barriers:
// four LDS stages of 2 x 64 keys x d x 2 B filled by direct-to-LDS copies (16 B per lane, no register
// staging) two tiles ahead, one s_waitcnt vmcnt + one s_barrier per tile.  Stage s holds K tile s+2
// and V tile s: exactly what iteration s+1 reads.  Barrier j makes the stages up to j visible (one
// more than iteration j reads, so the last tile's U needs no barrier of its own) and frees the slot
// of stage j-2 for the copies of stage j+2, which go out one at a time behind MFMAs of the pass.
//
// Register layout (as in the two-group kernel): scores are computed transposed, S^T = K Q^T, with
// the 32x32x16 MFMA; a lane owns one query and 16 of the 32 keys of a block, the other 16 sit in
// lane^32; the packed probabilities already are the B operand of O^T += V^T P^T; V^T fragments come
// through the transposing 64-bit LDS read.

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "attn_launch.h"
#include "gfx950_prims.h"
#include "launch_once.h"
#include "tile_schedule.h"

namespace {

// LDS fragments requested ahead of their MFMAs inside a pass (each fragment feeds MB MFMAs).
#ifndef ATTNP_FWIN
#define ATTNP_FWIN 3
#endif
// 1: the vector work of C_j is issued in slices between the MFMAs; 0: as one block after them.
#ifndef ATTNP_INTERLEAVE
#define ATTNP_INTERLEAVE 1
#endif
// 1: steady-state copies go out one by one behind MFMAs of the pass; 0: as a block after the barrier.
#ifndef ATTNP_COPIES_IN_PASS
#define ATTNP_COPIES_IN_PASS 1
#endif
// 1: with four waves of 64 rows the steady state runs in the generated assembly loop (attn_mb2_loop.inc); 0: in C++.
#ifndef ATTNP_ASM_LOOP
#define ATTNP_ASM_LOOP 1
#endif
#ifdef ATTNP_TIMING
// Profiling builds only: cycle and wall-clock totals of the main loop of the first workgroups.
constexpr int DBGP_WGS = 1024, DBGP_SLOTS = 8;
__device__ unsigned long long attnp_dbg[DBGP_WGS * 8 * DBGP_SLOTS];
#endif

// Compile-time loop: f(integral_constant<int, B>), ..., f(integral_constant<int, E - 1>).  Every register
// array below is indexed with such constants only (indices that merely become constant after loop
// unrolling leave the arrays in scratch memory).
template <int B, int E, typename F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (B < E) {
        f(std::integral_constant<int, B>{});
        static_for<B + 1, E>(f);
    }
}

// The lane id, recomputed where it is needed (two instructions).  The per-lane address offsets below are a few
// more instructions on top of it; derived afresh in every pass they never live across a pass, whereas held in
// registers for the whole kernel the register allocator spills them and reloads them in the main loop, each
// reload with a wait for ALL outstanding memory operations, the global -> LDS copies included.
__device__ __forceinline__ int fresh_lane() {
    int l;
    asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(l));
    return l;
}

// Exchange with lane^32 (see the two-group kernel: inline asm because the builtin's two results are
// folded into one when both inputs are the same value).
__device__ __forceinline__ float pipe_xor32_max(float x) {
    float a = x, b = x;
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
    return __builtin_fmaxf(a, b);
}
__device__ __forceinline__ float pipe_xor32_sum(float x) {
    float a = x, b = x;
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
    return a + b;
}

// The steady-state loop of the 64-rows-per-wave form as hand-scheduled assembly (gen_attn_mb2_loop.py writes it and
// documents its register contract).
#include "attn_mb2_loop.inc"

typedef float f32x32 __attribute__((ext_vector_type(32)));
typedef float f32x4v __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef int i32x16 __attribute__((ext_vector_type(16)));
typedef int i32x32 __attribute__((ext_vector_type(32)));

__device__ __forceinline__ f32x32 cat32(f32x16 a, f32x16 b) {
    return __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15, 16, 17, 18, 19, 20, 21, 22, 23, 24, 25, 26, 27, 28, 29, 30, 31);
}
__device__ __forceinline__ f32x16 lo16(f32x32 x) { return __builtin_shufflevector(x, x, 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15); }
__device__ __forceinline__ f32x16 hi16(f32x32 x) { return __builtin_shufflevector(x, x, 16, 17, 18, 19, 20, 21, 22, 23, 24, 25, 26, 27, 28, 29, 30, 31); }
__device__ __forceinline__ i32x32 cat8x4(const s16x8* f) {       // eight 4-register fragments -> one 32-register tuple
    i32x4 w[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) w[i] = __builtin_bit_cast(i32x4, f[i]);
    const i32x8 a = __builtin_shufflevector(w[0], w[1], 0, 1, 2, 3, 4, 5, 6, 7), b = __builtin_shufflevector(w[2], w[3], 0, 1, 2, 3, 4, 5, 6, 7);
    const i32x8 c = __builtin_shufflevector(w[4], w[5], 0, 1, 2, 3, 4, 5, 6, 7), d = __builtin_shufflevector(w[6], w[7], 0, 1, 2, 3, 4, 5, 6, 7);
    const i32x16 ab = __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15);
    const i32x16 cd = __builtin_shufflevector(c, d, 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15);
    return __builtin_shufflevector(ab, cd, 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15, 16, 17, 18, 19, 20, 21, 22, 23, 24, 25, 26, 27, 28, 29, 30, 31);
}

template <int DTYPE, int D, int NW, int MB, bool CAUSAL>
__global__ __launch_bounds__(NW * 64)
void attn_fwd_pipe_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
                          uint16_t* __restrict__ o, float* __restrict__ lse, int N, int nqt, int total,
                          float scale, float scale_log2e)
{
    typedef Elem<DTYPE> E;
    constexpr int BN = 64, STAGES = 4, AHEAD = 2;
    constexpr int BM = NW * MB * 32;            // query rows per workgroup
    constexpr int KB = BN / 32;                 // 32-key blocks per K/V tile
    constexpr int KK = D / 16;                  // contraction steps of Q K^T
    constexpr int DB = D / 32;                  // 32-wide feature blocks of O
    constexpr int ROW_BYTES = D * 2;
    constexpr int TILE_BYTES = BN * ROW_BYTES;  // one K or one V tile
    constexpr int STAGE_BYTES = 2 * TILE_BYTES;
    constexpr int RB = BN / 16;                 // 16-row blocks per tile
    constexpr int CHUNKS = TILE_BYTES / 1024;   // 1 KiB wave-transfers per tile
    constexpr int CPW = CHUNKS / NW;            // ... per wave
    constexpr int LPG = 2 * CPW;                // copies a wave issues per stage (K pieces, then V pieces)
    static_assert(CHUNKS % NW == 0 && CPW >= 1, "a tile must split evenly over the waves");
    static_assert(BN % (MB * 32) == 0, "only a wave's last tile may need a mask");
    constexpr bool ASM_LOOP = MB == 2 && NW == 4 && D == 128 && ATTNP_ASM_LOOP;   // the steady state as the generated assembly loop

    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const unsigned lds_base = (unsigned)(size_t)(LDS_AS void*)smem;

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int lr = lane & 31, g = lane >> 5;

    // ---- which (batch*head, query tile) this workgroup works on
    const int tile = __builtin_amdgcn_readfirstlane(tile_schedule(total, (int)gridDim.x, (int)blockIdx.x, 0));
    const int bh = __builtin_amdgcn_readfirstlane(tile / nqt);
    int qt = tile - bh * nqt;
    if (CAUSAL) qt = nqt - 1 - qt;              // long rows first
    const int q0 = qt * BM;
    const int wq0 = __builtin_amdgcn_readfirstlane(q0 + wave * (MB * 32));   // first query row of this wave
    const size_t head_off = (size_t)bh * N * D;
    const uint16_t* qh = q + head_off;
    const char* kh = uniform_ptr(reinterpret_cast<const char*>(k + head_off));
    const char* vh = uniform_ptr(reinterpret_cast<const char*>(v + head_off));
    int nt = (N + BN - 1) / BN;                 // K/V tiles the workgroup walks
    if (CAUSAL) nt = min(nt, (min(q0 + BM, N) - 1) / BN + 1);
    int nt_w = nt;                              // those this wave computes on (1 <= nt_w <= nt)
    if (CAUSAL) nt_w = min(nt, (wq0 + MB * 32 - 1) / BN + 1);
    nt = __builtin_amdgcn_readfirstlane(nt);
    nt_w = __builtin_amdgcn_readfirstlane(nt_w);
    const int last_stage = max(AHEAD - 1, nt - 1);   // stages -2 .. last_stage are copied

    // ---- global -> LDS copies.  A tile is CHUNKS pieces of 1 KiB; piece wc = (feature group wc / RB,
    // 16-row block wc % RB) is a (16 rows x 64 B) block of the source.
    // K tile in LDS: [feature group of 32][16-row block][16-byte column of the group (4)][row (16)][16 B]
    // V tile in LDS: [feature group of 32][row (BN)][64 B]
    // Lane L of a K piece fetches row L%16, column L/16 of the block; of a V piece row L/4, column L%4.
    auto k_copy_off = [&](int ln) __attribute__((always_inline)) -> unsigned { return (ln & 15) * ROW_BYTES + (ln >> 4) * 16; };
    auto v_copy_off = [&](int ln) __attribute__((always_inline)) -> unsigned { return (ln >> 2) * ROW_BYTES + (ln & 3) * 16; };
    int piece_src[CPW], piece_dst[CPW];         // wave-uniform: source offset inside a tile, LDS offset inside a K or V slot
#pragma unroll
    for (int i = 0; i < CPW; ++i) {
        const int wc = wave * CPW + i, fg = wc / RB, rb = wc % RB;
        piece_src[i] = rb * 16 * ROW_BYTES + fg * 64;
        piece_dst[i] = wc * 1024;
    }
    // Tile t is copied from the 64 rows starting at tile_row(t) = min(t * BN, N - BN): a tile that overhangs
    // the end of the sequence (the ragged last one, or one past the end that is only copied to keep the wait
    // counts uniform) is shifted back so that it ends with the sequence.  Every copy then reads whole rows that
    // exist, with scalar address arithmetic only; the softmax of the ragged tile masks the keys the shift
    // brought in again (softmax_mask).  Sequences shorter than one tile (a single, clamped tile) take
    // issue_stage's per-lane path instead.
    auto tile_row = [&](int t) __attribute__((always_inline)) -> int { return max(min(t * BN, N - BN), 0); };
    // copy i of stage s: K piece i < CPW (of K tile s + 2), else V piece i - CPW (of V tile s)
    auto issue_piece = [&](int s, auto ic, unsigned koff, unsigned voff) __attribute__((always_inline)) {
        constexpr int i = decltype(ic)::value;
        const unsigned sbase = lds_base + ((s + 2 * STAGES) % STAGES) * STAGE_BYTES;
        if constexpr (i < CPW) dma16(kh + (size_t)tile_row(s + 2) * ROW_BYTES + piece_src[i], koff, sbase + piece_dst[i]);
        else dma16(vh + (size_t)tile_row(s) * ROW_BYTES + piece_src[i - CPW], voff, sbase + TILE_BYTES + piece_dst[i - CPW]);
    };
    // all copies of stage s as one block
    auto issue_stage = [&](int s) __attribute__((always_inline)) {
        const unsigned sbase = lds_base + ((s + 2 * STAGES) % STAGES) * STAGE_BYTES;
        const int lane = fresh_lane();
        if (N >= BN) {
            const unsigned koff = k_copy_off(lane), voff = v_copy_off(lane);
            static_for<0, LPG>([&](auto ic) __attribute__((always_inline)) { issue_piece(s, ic, koff, voff); });
        } else {                                // rows clamped into the sequence (surplus rows are masked)
#pragma unroll
            for (int i = 0; i < CPW; ++i) {
                const int wc = wave * CPW + i, fg = wc / RB, rb = wc % RB;
                const int row = min(rb * 16 + (lane & 15), N - 1);
                dma16(kh, (unsigned)(row * ROW_BYTES + fg * 64 + (lane >> 4) * 16), sbase + piece_dst[i]);
            }
#pragma unroll
            for (int i = 0; i < CPW; ++i) {
                const int wc = wave * CPW + i, fg = wc / RB, rb = wc % RB;
                const int row = min(rb * 16 + (lane >> 2), N - 1);
                dma16(vh, (unsigned)(row * ROW_BYTES + fg * 64 + (lane & 3) * 16), sbase + TILE_BYTES + piece_dst[i]);
            }
        }
    };

    // ---- prologue: the whole ring in flight, then the Q fragments into registers.  The Q loads are ordinary
    // loads issued AFTER the copies, followed by a wait for everything: the compiler must know that their
    // destination registers are busy until the data is there.  (Loads hidden in asm statements would let it
    // move or reuse those registers while the loads are still in flight: with 64 rows per wave it did, and a
    // late Q fragment landed in the register that held a copy's address offset.)
#pragma unroll
    for (int s0 = -2; s0 < AHEAD; ++s0) issue_stage(s0);
    s16x8 Qf[MB][KK];                           // B operand of T: query lane%32, features (kk*2 + lane/32)*8 .. +7
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const int row = min(wq0 + mb * 32 + lr, N - 1);
        const uint16_t* qr = qh + (size_t)row * D + g * 8;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) Qf[mb][kk] = *reinterpret_cast<const s16x8*>(qr + kk * 16);
    }

    f32x16 O[MB][DB], S[2][MB][KB];
    unsigned pw[MB][KB * 8];                    // P as packed 16-bit pairs: one buffer, rewritten word by word behind the U that reads it
    float m_run[MB], l_run[MB], negmc[MB];      // reference maximum (raw dot-product units), row sum, -m * scale * log2 e

    // per-lane LDS read offsets (the rest of every address is an immediate)
    auto k_read_off = [&](int ln) __attribute__((always_inline)) -> int { return ((ln >> 4) & 1) * 1024 + (ln >> 5) * 256 + (ln & 15) * 16; };
    auto v_read_off = [&](int ln) __attribute__((always_inline)) -> int {
        return TILE_BYTES + (4 * (ln >> 5) + ((ln & 15) >> 2)) * 64 + ((ln >> 4) & 1) * 32 + (ln & 3) * 8;
    };
    // K fragment (A operand of T): keys kb*32 + lane%32, features (kk*2 + lane/32)*8 .. +7
    auto read_kf = [&](const char* sk, int kb, int kk) __attribute__((always_inline)) -> s16x8 {
        return *reinterpret_cast<const s16x8*>(sk + ((kk >> 1) * RB + kb * 2) * 1024 + (kk & 1) * 512);
    };
    // V^T fragment (A operand of U): features db*32 + lane%32, the 8 keys of block kb that the P operand
    // of step ks holds in this lane group, through the transposing LDS read
    auto read_vf = [&](const char* sv, int kb, int ks, int db) __attribute__((always_inline)) -> s16x8 {
        const char* a = sv + db * (BN * 64) + (kb * 32 + ks * 16) * 64;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(a));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(a + 8 * 64));
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    };

    // ---- C of one tile.
    // Steady state ("fast" path): the reference of the exponentials is left where it is,
    // p = exp2(s*c - m*c) with the m the row had when it was last set; round, pack, add to the tile's row sum.
    // No row maximum and no cross-lane step.  What can go wrong is a score far above the reference: its 16-bit
    // probability would overflow.  The row sum tells: if a lane's sum over the tile is <= FAST_SUM_MAX, none of
    // its probabilities was larger.  Otherwise (or when the sum is not a number: on the first tile the
    // reference is still +inf) the tile is redone on the slow path, which moves the reference to the running
    // maximum.  The reference is always a maximum the row has really seen, so the largest probability of a row
    // is never below 1 and nothing underflows that matters.
    // The fast path is cut into units: unit k of a 32-query block holds the two exponentials of score pair k
    // (scale-and-subtract FMA, then exp2; two independent chains), the rounding and packing of pair k-1 and the
    // row-sum update of pair k-2 (a dependent vector instruction issues a cycle or two late; a unit apart, none waits).
    constexpr int PAIRS = KB * 8;               // score pairs per lane and 32-query block
    constexpr int FUNITS = PAIRS + 1, NUNITS = MB * FUNITS;
    constexpr int NCH = 2;                      // accumulation chains of a row sum
    constexpr float FAST_SUM_MAX = 16384.0f;
    float fb[MB][2], sm_sum[MB][NCH];
    auto softmax_mask = [&](auto par, int j) __attribute__((always_inline)) {
        constexpr int P = decltype(par)::value;
        const int kv0 = tile_row(j), first = j * BN;   // the tile's first row and the first key not yet seen
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            const int qi = wq0 + mb * 32 + lr;
            const int lim = CAUSAL ? min(qi, N - 1) : N - 1;   // last visible key
#pragma unroll
            for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int key = kv0 + kb * 32 + (i >> 2) * 8 + g * 4 + (i & 3);
                    if (key > lim || key < first) S[P][mb][kb][i] = -__builtin_inff();
                }
        }
    };
    auto fast_unit = [&](auto par, auto uc) __attribute__((always_inline)) {
        constexpr int P = decltype(par)::value;
        constexpr int u = decltype(uc)::value, k = u / MB, mb = u % MB;   // the blocks take turns
        if constexpr (k >= 1 && k - 1 < PAIRS) {    // word k-1 of the block's P, and its two probabilities into the row sum
            unsigned wd = E::pack2(fb[mb][0], fb[mb][1]);
            // (pins the word where it is written: it is only used by the next pass, and the compiler would
            // otherwise sink the conversion down to that use)
            asm volatile("" : "+v"(wd));
            pw[mb][k - 1] = wd;
            // (vector additions, not a v_dot2c on the packed pair: see Elem::add_pair_valu; two chains)
            float s0 = E::add_pair_valu(wd, fb[mb][0], fb[mb][1], k - 1 < NCH ? 0.f : sm_sum[mb][(k - 1) % NCH]);
            asm volatile("" : "+v"(s0));        // (left alone the compiler collects all row-sum updates at the end of the loop body)
            sm_sum[mb][(k - 1) % NCH] = s0;
        }
        if constexpr (k < PAIRS) {              // the exponentials of pair k
            constexpr int kb = k / 8, t = k % 8;
            float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(S[P][mb][kb][2 * t], scale_log2e, negmc[mb]));
            float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(S[P][mb][kb][2 * t + 1], scale_log2e, negmc[mb]));
            asm volatile("" : "+v"(p0), "+v"(p1));
            fb[mb][0] = p0;
            fb[mb][1] = p1;
        }
    };
    // The slow path: row maximum (one lane <-> lane+32 exchange), reference moved to the running maximum, O
    // and the running row sum rescaled, the tile's probabilities and row sum computed afresh.  Runs after the
    // pass's last MFMA (it rewrites P and O).  Also the path of a wave's last tile, which may carry a mask.
    auto slow_softmax = [&](auto par) __attribute__((always_inline)) {
        constexpr int P = decltype(par)::value;
#ifdef ATTNP_X_NOSLOW
        return;
#endif
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            float mx = S[P][mb][0][0];
#pragma unroll
            for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                for (int i = 0; i < 16; ++i) mx = __builtin_fmaxf(mx, S[P][mb][kb][i]);
            mx = pipe_xor32_max(mx);
            const float m_old = m_run[mb];
            const float m_new = __builtin_fmaxf(m_old, mx);
            const float alpha = m_old == -__builtin_inff() ? 0.f : __builtin_amdgcn_exp2f((m_old - m_new) * scale_log2e);
            const float nm = -m_new * scale_log2e;
            m_run[mb] = m_new;
            negmc[mb] = nm;
            float ts[2] = {0.f, 0.f};
#pragma unroll
            for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                for (int t = 0; t < 8; ++t) {
                    const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(S[P][mb][kb][2 * t], scale_log2e, nm));
                    const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(S[P][mb][kb][2 * t + 1], scale_log2e, nm));
                    const unsigned wd = E::pack2(p0, p1);
                    pw[mb][kb * 8 + t] = wd;
                    ts[t % 2] = E::add_pair_valu(wd, p0, p1, ts[t % 2]);
                    __builtin_amdgcn_sched_barrier(0);   // (a rare path: kept narrow, so that it claims no registers of its own)
                }
            l_run[mb] = __builtin_fmaf(l_run[mb], alpha, ts[0] + ts[1]);
            // whole-vector multiplies (element-wise updates would make the compiler split the accumulator tuples),
            // one block at a time, so that this rare path does not claim registers the steady state needs
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                O[mb][db] = O[mb][db] * alpha;
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };
    // End of the fast path: the tile's row sums and the overflow test.  Returns true (wave-uniform) when the tile
    // has to be redone on the slow path; the running sums are only updated when it does not.
    auto fast_finish = [&]() __attribute__((always_inline)) -> bool {
        float ts[MB];
        bool bad = false;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            ts[mb] = sm_sum[mb][0];
#pragma unroll
            for (int c = 1; c < NCH; ++c) ts[mb] += sm_sum[mb][c];
            bad |= !(ts[mb] <= FAST_SUM_MAX);
        }
        if (__builtin_amdgcn_ballot_w64(bad) != 0) return true;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) l_run[mb] += ts[mb];
        return false;
    };

    // ---- one pass over a stage: the MFMAs of T (S^T of parity PAR^1 = K Q^T) and/or U (O^T += V^T P^T
    // with the P of parity PAR^1), LDS fragments requested FWIN fragments ahead, every fragment feeding
    // the MFMAs of the wave's MB query blocks in snake order (consecutive MFMAs share the fragment or
    // the Q/P operand), and between the MFMAs the units of C on the scores of parity PAR.  The
    // scheduling barriers keep that order.  `copies`: the pass also issues the copies of stage
    // j + AHEAD, one piece behind each of a few MFMAs (the sequence then holds at least one whole tile).
    // Returns whether C has to be redone on the slow path (always false without C).
    auto pass = [&](auto do_u, auto do_t, auto do_c, auto copies, auto par, const char* st, int j) __attribute__((always_inline)) -> bool {
        constexpr int P = decltype(par)::value;
        constexpr bool COPIES = decltype(copies)::value;
        constexpr bool C = decltype(do_c)::value;
        constexpr int NU = decltype(do_u)::value ? KB * 2 * DB : 0;    // U's fragments come first
        constexpr int NT = decltype(do_t)::value ? KB * KK : 0;
        constexpr int NF = NT + NU, NM = NF * MB;
        constexpr int FWIN = ATTNP_FWIN < NF ? ATTNP_FWIN : NF;
        constexpr bool IL = C && ATTNP_INTERLEAVE;
        constexpr int CSTRIDE = NM / LPG > 0 ? NM / LPG : 1;           // a copy behind every CSTRIDE-th MFMA
        const int pl = fresh_lane();
        const char* sk = st + k_read_off(pl);
        const char* sv = st + v_read_off(pl);
        const unsigned koff = COPIES ? k_copy_off(pl) : 0u, voff = COPIES ? v_copy_off(pl) : 0u;
        s16x8 fr[NF > 0 ? NF : 1];
        auto fetch = [&](auto fc) __attribute__((always_inline)) {
            constexpr int f = decltype(fc)::value;
            if constexpr (f < NU) fr[f] = read_vf(sv, f / (2 * DB), (f / DB) % 2, f % DB);
            else fr[f] = read_kf(sk, (f - NU) % KB, (f - NU) / KB);
        };
        auto run_mfma = [&](auto fc, auto mbc) __attribute__((always_inline)) {
            constexpr int f = decltype(fc)::value, mb = decltype(mbc)::value;
            if constexpr (f >= NU) {
                constexpr int kb = (f - NU) % KB, kk = (f - NU) / KB;
                if constexpr (kk == 0) S[P ^ 1][mb][kb] = E::mfma(fr[f], Qf[mb][kk], f32x16(0.f));
                else S[P ^ 1][mb][kb] = E::mfma(fr[f], Qf[mb][kk], S[P ^ 1][mb][kb]);
            } else {
                constexpr int kb = f / (2 * DB), ks = (f / DB) % 2, db = f % DB;
                u32x4 w;
                w[0] = pw[mb][kb * 8 + ks * 4 + 0];
                w[1] = pw[mb][kb * 8 + ks * 4 + 1];
                w[2] = pw[mb][kb * 8 + ks * 4 + 2];
                w[3] = pw[mb][kb * 8 + ks * 4 + 3];
                O[mb][db] = E::mfma(fr[f], __builtin_bit_cast(s16x8, w), O[mb][db]);
            }
        };
        static_for<0, FWIN>([&](auto fc) __attribute__((always_inline)) { fetch(fc); });
        static_for<0, NF>([&](auto fc) __attribute__((always_inline)) {
            constexpr int f = decltype(fc)::value;
            if constexpr (f + FWIN < NF) fetch(std::integral_constant<int, f + FWIN>{});
            static_for<0, MB>([&](auto ic) __attribute__((always_inline)) {
                constexpr int i = decltype(ic)::value, m = f * MB + i;
                run_mfma(fc, std::integral_constant<int, (f & 1) ? MB - 1 - i : i>{});
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (COPIES) {
                    static_for<0, LPG>([&](auto cc) __attribute__((always_inline)) {
                        constexpr int c = decltype(cc)::value;
                        if constexpr (m == 1 + c * CSTRIDE || (1 + c * CSTRIDE >= NM && m == NM - 1)) issue_piece(j + AHEAD, cc, koff, voff);
                    });
                    __builtin_amdgcn_sched_barrier(0);
                }
                if constexpr (IL) {
                    // the units are spread evenly over the MFMAs from USTART on
                    constexpr int USTART = NU > 0 ? DB * MB - 2 : 0, NS = NM - USTART;
                    if constexpr (m >= USTART) {
                        constexpr int mm = m - USTART;
                        static_for<(mm * NUNITS + NS - 1) / NS, ((mm + 1) * NUNITS + NS - 1) / NS>(
                            [&](auto uc) __attribute__((always_inline)) {
                                // a word of P may only be rewritten after the last MFMA of U that reads the old one:
                                // words 4g .. 4g+3 of every block are read by MFMAs g*DB*MB .. (g+1)*DB*MB - 1
                                constexpr int u = decltype(uc)::value, q = u / MB - 1;
                                static_assert(NU == 0 || q < 0 || q >= PAIRS || m >= (q / 4 + 1) * DB * MB - 1,
                                              "P word rewritten before U has read it");
                                fast_unit(par, uc);
                            });
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            });
        });
        if constexpr (C && !IL) {
            static_for<0, NUNITS>([&](auto uc) __attribute__((always_inline)) { fast_unit(par, uc); });
        }
        if constexpr (C) return fast_finish();
        else return false;
    };

    // Barrier j: every wave's share of the stages up to j has landed (the copies of stage j+1 may still
    // be in flight) and nobody reads stage j-2 any more, so that slot takes the copies of stage j+AHEAD.
    auto step = [&](int j, bool with_copies = true) __attribute__((always_inline)) {
        if (j + 1 <= last_stage) wait_vmcnt<LPG>(); else wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();
        const int s = j + AHEAD;
        if (with_copies && s <= last_stage) issue_stage(s);
    };
    auto stage_ptr = [&](int s) __attribute__((always_inline)) -> const char* { return smem + ((s + 2 * STAGES) % STAGES) * STAGE_BYTES; };

    // Use the Q fragments once here: the compiler then waits for their loads now (its vmcnt(0) also covers the
    // copies of all four stages issued before them) instead of inside the first pass.
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) asm volatile("" :: "v"(Qf[mb][kk]));
    wait_vmcnt<0>();
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        m_run[mb] = -__builtin_inff();
        l_run[mb] = 0.f;
        negmc[mb] = __builtin_inff();           // no reference yet: the first tile takes the slow path
#pragma unroll
        for (int db = 0; db < DB; ++db) O[mb][db] = f32x16(0.f);
#pragma unroll
        for (int t = 0; t < KB * 8; ++t) pw[mb][t] = 0u;
    }
    __builtin_amdgcn_s_barrier();               // stages -2 .. 0 are complete for every wave
#ifdef ATTNP_TIMING
    const unsigned long long rt0 = __builtin_amdgcn_s_memrealtime(), ct0 = __builtin_readcyclecounter();
#endif

    constexpr std::integral_constant<int, 0> P0{};
    constexpr std::integral_constant<int, 1> P1{};
    constexpr std::true_type Y{};
    constexpr std::false_type NO{};
    constexpr std::integral_constant<bool, ATTNP_COPIES_IN_PASS != 0> CIP{};

    // Iteration j of a wave (after barrier j; it reads stage j-1 = K tile j+1 and V tile j-1):
    //   j <= nt_w - 2   MFMAs of T_{j+1} and U_{j-1}, C_j in between (no tile before a wave's last needs a mask)
    //   j == nt_w - 1   U_{j-1}, then C_j with the mask (diagonal or ragged end), then U_j (stage j is visible)
    //   j >= nt_w       nothing: the wave only keeps copying its share for the others
    pass(NO, Y, NO, NO, P1, stage_ptr(-2), 0);                          // T_0 into the scores of parity 0
    int j = 0;
    if (nt_w >= 2) {
        step(0);
        pass(NO, Y, NO, NO, P0, stage_ptr(-1), 0);                      // T_1
        slow_softmax(P0);                                               // C_0 sets the reference
        j = 1;
        // The steady state: two iterations per trip of the inner loop (scores of alternating parity), copies
        // issued inside the passes, the fast softmax only.  A tile whose probabilities overflowed leaves the
        // loop, is redone on the slow path out here, and the loop of the matching phase is entered again.
        // (The mask never applies here: N >= BN because nt_w >= 2, and only a wave's last tile is ragged or diagonal.)
        while (j <= nt_w - 2) {
            int redo = -1;                      // parity of a tile to redo
            if (ASM_LOOP && (j & 1)) {
#if defined(__HIP_DEVICE_COMPILE__)
                f32x32 o0 = cat32(O[0][0], O[0][1]), o1 = cat32(O[0][2], O[0][3]), o2 = cat32(O[MB - 1][0], O[MB - 1][1]), o3 = cat32(O[MB - 1][2], O[MB - 1][3]);
                f32x32 s0 = cat32(S[0][0][0], S[0][0][1]), s1 = cat32(S[0][MB - 1][0], S[0][MB - 1][1]);
                f32x32 s2 = cat32(S[1][0][0], S[1][0][1]), s3 = cat32(S[1][MB - 1][0], S[1][MB - 1][1]);
                const i32x32 q0 = cat8x4(Qf[0]), q1 = cat8x4(Qf[MB - 1]);
                i32x32 pv;
#pragma unroll
                for (int i = 0; i < 32; ++i) pv[i] = (int)pw[(i / 16) % MB][i % 16];
                f32x4v st = {negmc[0], negmc[MB - 1], l_run[0], l_run[MB - 1]};
                const int ln = fresh_lane();
                const int krd = k_read_off(ln), vrd = v_read_off(ln);
                const unsigned kcp = k_copy_off(ln), vcp = v_copy_off(ln);
                int jj = j, flag;
                const int j_end = nt_w - 2;
#define ATTN_MB2_OPERANDS \
                    : "+{a[0:31]}"(o0), "+{a[32:63]}"(o1), "+{a[64:95]}"(o2), "+{a[96:127]}"(o3), \
                      "+{v[0:31]}"(s0), "+{v[32:63]}"(s1), "+{v[64:95]}"(s2), "+{v[96:127]}"(s3), \
                      "+{v[128:159]}"(pv), "+{v[160:163]}"(st), "+{s40}"(jj), "={s46}"(flag) \
                    : "{a[128:159]}"(q0), "{a[160:191]}"(q1), "{s[36:37]}"(kh), "{s[38:39]}"(vh), "{s41}"(j_end), "{s42}"(scale_log2e), \
                      "{s43}"(lds_base), "{s44}"(wave), "{s45}"(N), "{v200}"(krd), "{v201}"(vrd), "{v202}"(kcp), "{v203}"(vcp) \
                    : ATTN_MB2_LOOP_CLOBBERS
                if constexpr (DTYPE == 0) asm volatile(ATTN_MB2_LOOP_F16 ATTN_MB2_OPERANDS);
                else asm volatile(ATTN_MB2_LOOP_BF16 ATTN_MB2_OPERANDS);
#undef ATTN_MB2_OPERANDS
                O[0][0] = lo16(o0); O[0][1] = hi16(o0); O[0][2] = lo16(o1); O[0][3] = hi16(o1);
                O[MB - 1][0] = lo16(o2); O[MB - 1][1] = hi16(o2); O[MB - 1][2] = lo16(o3); O[MB - 1][3] = hi16(o3);
                S[0][0][0] = lo16(s0); S[0][0][1] = hi16(s0); S[0][MB - 1][0] = lo16(s1); S[0][MB - 1][1] = hi16(s1);
                S[1][0][0] = lo16(s2); S[1][0][1] = hi16(s2); S[1][MB - 1][0] = lo16(s3); S[1][MB - 1][1] = hi16(s3);
#pragma unroll
                for (int i = 0; i < 32; ++i) pw[(i / 16) % MB][i % 16] = (unsigned)pv[i];
                negmc[0] = st[0]; negmc[MB - 1] = st[1]; l_run[0] = st[2]; l_run[MB - 1] = st[3];
                j = jj;
                if (flag) redo = j & 1;
#endif
            } else if ((j & 1) && j + 1 <= nt_w - 2) {
                do {                            // bottom-tested: the accumulators are updated in place
                    step(j, !ATTNP_COPIES_IN_PASS);
                    if (__builtin_expect(pass(Y, Y, Y, CIP, P1, stage_ptr(j - 1), j), 0)) { redo = 1; break; }
                    step(j + 1, !ATTNP_COPIES_IN_PASS);
                    if (__builtin_expect(pass(Y, Y, Y, CIP, P0, stage_ptr(j), j + 1), 0)) { redo = 0; ++j; break; }
                    j += 2;
                } while (j + 1 <= nt_w - 2);
            } else {
                step(j, !ATTNP_COPIES_IN_PASS);
                if (j & 1) { if (pass(Y, Y, Y, CIP, P1, stage_ptr(j - 1), j)) redo = 1; }
                else { if (pass(Y, Y, Y, CIP, P0, stage_ptr(j - 1), j)) redo = 0; }
                if (redo < 0) ++j;
            }
            // (the scores of the tile are still in their registers: the other parity's were written meanwhile)
            if (redo == 1) { slow_softmax(P1); ++j; }
            else if (redo == 0) { slow_softmax(P0); ++j; }
        }
    }
    // j == nt_w - 1: the last tile this wave computes on
    auto tail = [&](auto par, auto parx) __attribute__((always_inline)) {
        step(j);
        if (j >= 1) pass(Y, NO, NO, NO, par, stage_ptr(j - 1), j);      // U_{j-1}
        softmax_mask(par, j);
        slow_softmax(par);
        pass(Y, NO, NO, NO, parx, stage_ptr(j), j + 1);                 // U_j
    };
#ifdef ATTNP_X_ONETAIL
    tail(P1, P0);
#else
    if (j & 1) tail(P1, P0); else tail(P0, P1);
#endif
    for (++j; j < nt; ++j) step(j);             // idle tail of a causal wave
    wait_vmcnt<0>();

    // ---- epilogue: normalise, write O (16-bit) and LSE (natural log)
    {
        uint16_t* oh = o + head_off;
        float* lh = lse + (size_t)bh * N;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            const float l_tot = pipe_xor32_sum(l_run[mb]);
            const float inv = 1.0f / l_tot;
            const int row = wq0 + mb * 32 + lr;
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
    }
#ifdef ATTNP_TIMING
    if (blockIdx.x < DBGP_WGS && lane == 0) {
        unsigned long long* d = attnp_dbg + (blockIdx.x * 8 + wave) * DBGP_SLOTS;
        d[5] = nt;
        d[6] = __builtin_amdgcn_s_memrealtime() - rt0;   // 100 MHz ticks
        d[7] = __builtin_readcyclecounter() - ct0;
    }
#endif
}

template <int DTYPE, int D, int NW, int MB, bool CAUSAL>
int launch_pipe(const AttnLaunchArgs& a)
{
    constexpr int BM = NW * MB * 32;
    constexpr int smem = 4 * 2 * 64 * D * 2;
    auto kern = attn_fwd_pipe_kernel<DTYPE, D, NW, MB, CAUSAL>;
    static PerDeviceOnce once;                  // the attribute belongs to the (kernel, device) pair
    if (once.prepare(reinterpret_cast<const void*>(kern), smem) < 0) return -1;
    const int nqt = (a.N + BM - 1) / BM;
    const long long total = (long long)nqt * a.B * a.H;
    const float log2e = 1.4426950408889634f;
    const uint16_t* q = (const uint16_t*)a.q;
    const uint16_t* k = (const uint16_t*)a.k;
    const uint16_t* v = (const uint16_t*)a.v;
    uint16_t* o = (uint16_t*)a.o;
    float* lse = a.lse;
    int N = a.N, nqt_arg = nqt, total_arg = (int)total;
    float scale = a.scale, scale_log2e = a.scale * log2e;
    void* args[] = {&q, &k, &v, &o, &lse, &N, &nqt_arg, &total_arg, &scale, &scale_log2e};
    const hipError_t e = hipLaunchKernel(reinterpret_cast<const void*>(kern), dim3((unsigned)total), dim3(NW * 64),
                                         args, smem, (hipStream_t)a.stream);
    return e == hipSuccess ? 0 : -1;
}

}  // namespace

#ifdef ATTNP_TIMING
extern "C" int attnp_dbg_read(unsigned long long* host, int n)
{
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(attnp_dbg), sizeof(unsigned long long) * n);
}
#endif

// The in-wave pipelined kernel for d = 128 (query rows per workgroup: 256 either way).
int attn_pipe_launch(const AttnLaunchArgs& a)
{
    constexpr int NW = ATTNP_CFG_NW, MB = 8 / ATTNP_CFG_NW;
    if (a.d != 128) return -1;
#ifdef ATTNP_DEV_ONE   // (development builds: one instantiation only)
    return launch_pipe<0, 128, NW, MB, false>(a);
#else
    if (a.dtype == 0) return a.causal ? launch_pipe<0, 128, NW, MB, true>(a) : launch_pipe<0, 128, NW, MB, false>(a);
    return a.causal ? launch_pipe<1, 128, NW, MB, true>(a) : launch_pipe<1, 128, NW, MB, false>(a);
#endif
}
