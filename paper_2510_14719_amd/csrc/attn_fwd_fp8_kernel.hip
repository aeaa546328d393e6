// Fused attention forward for gfx950 (MI355X) on 8-bit-float inputs: Q, K, V in OCP E4M3, O in
// fp16 or bf16, per-row log-sum-exp in fp32.  The paper evaluates attention in a second precision
// it calls FP8 (Section 5.4); the three stages per key/value tile are the ones of Section 3.4.2
// (T = Q K^T on the matrix cores, C = softmax on the vector ALU, U = P V on the matrix cores).
//
// Schedule.  At this precision the vector ALU is the busier unit (the MFMA time halves, the
// softmax does not), and a 32x32x64 MFMA on 8-bit operands occupies the matrix pipe for 64 cycles
// while its wave is free to issue vector instructions (measured: 12 FMAs between two such MFMAs of
// one wave cost nothing).  So the coarse-grained pipeline of the paper's Algorithm 1 lives INSIDE
// every wave's instruction stream here: in iteration j a wave issues the MFMAs of U_{j-1} and
// T_{j+1} and, between them, slices of the softmax C_j.  S and P are double buffered in registers
// (tile parity), the loop is unrolled by two.  All eight waves run the same code; the two waves of
// a SIMD fill each other's gaps on both pipes.
//
// Data movement.  A ring of LDS stages (four by default; a stage is 16 KiB at d = 128), filled by
// direct-to-LDS copies (16 B per lane, no register staging) STAGES - 2 tiles ahead; one s_waitcnt +
// one s_barrier per tile stand in for the full/empty credits of the paper's aref ring (Section
// 3.3): a stage is overwritten only after every wave has passed the barrier that follows its last
// read of it.  Stage s holds K tile s+2 and V tile s, the pair that iteration s+1 reads.  Barrier j
// makes stage j visible, one stage more than iteration j reads, so the last tile's U needs no
// barrier of its own.  In the steady state a wave issues its copies of a stage one by one behind
// the first MFMAs of the pass (+3 % over issuing them as a block after the barrier; a copy
// instruction holds its wave for 60-90 cycles, which a 64-cycle MFMA of the same wave covers).
// (Measured on MI355X: a deeper ring and requesting the next tile's first fragments before the
// barrier each cost 1-3 %; four waves of 32 query rows per workgroup instead of eight: -20 %.)
//
// What changes with the element type:
//  * Both contractions use the 32x32x64 MFMA on 8-bit operands (32 bytes per lane and operand):
//    T takes D/64 steps per 32-key block, U one step per 64 keys and 32 output features.
//  * The probabilities are rounded to E4M3 (round to nearest even) before the second contraction.
//    The softmax reference only moves when a row maximum grew by more than 2^8, so they stay
//    below 2^8 < 448 and never overflow the format.
//  * The row sum comes from the matrix cores as well: next to the D/32 feature blocks of V^T the
//    second contraction multiplies a block of ones with the same P operand, which yields the sum
//    of the ROUNDED probabilities of every query row (O is then an exact convex combination of the
//    V rows) and takes the additions off the vector ALU.
//  * LDS layouts.  A key row is D bytes, at most one 128-byte memory line, so every copy
//    instruction fetches whole rows (8 or 16 per instruction, fully coalesced) and both tiles are
//    row-major in the LDS; only the order of the 16-byte columns inside a row is permuted (which
//    global column a lane fetches is free, where its 16 bytes land is not):
//      K tile: row = key, column c stored at slot c ^ swK(row): the A operand of T (lane = key, 32
//              consecutive features = two 128-bit reads) is conflict free over 16 consecutive keys.
//      V tile: row = position, where position p holds the key with bits 2 and 3 of p swapped, and
//              column c stored at slot c ^ swV(p): the A operand of U (lane = feature, 8 keys per
//              read) comes from the transposing 64-bit read for 8-bit elements; the 8 keys of a
//              read are 8 consecutive positions, and a half-wave's 8 rows x 32 bytes cover all banks.
//
// Register layout: the scores are computed transposed (S^T = K Q^T), a lane owns one query and
// half of the keys of a 32-key block, the row maximum needs one lane <-> lane+32 exchange, and the
// packed probabilities already are the B operand of the second contraction.

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "attn_launch.h"
#include "gfx950_prims.h"
#include "launch_once.h"
#include "tile_schedule.h"

namespace {

typedef int i32x2 __attribute__((ext_vector_type(2)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x8 __attribute__((ext_vector_type(8)));

// The softmax reference moves only when a row maximum grew by more than this many powers of two
// (the largest probability then is 2^8 = 256, below the largest finite E4M3 value 448).
constexpr float RESCALE_LOG2_FP8 = 8.0f;

// LDS fragments requested ahead of their MFMA inside a pass.
#ifndef ATTN8_FWIN
#define ATTN8_FWIN 2
#endif

// 1: the softmax of tile j is issued in slices between the MFMAs of U_{j-1} and T_{j+1} (the
// software pipeline described above); 0: after them, as one block.
#ifndef ATTN8_INTERLEAVE
#define ATTN8_INTERLEAVE 1
#endif

// 1: the causal launch is persistent (one workgroup per CU walking the static serpentine tile schedule, tile after
// tile with a barrier in between).  Measured on MI355X (B2 H32 N8192 d128 causal): 1626 TFLOP/s against 1683 with one
// workgroup per tile: the hardware's own dispatch already overlaps one workgroup's epilogue with the next one's
// prologue, which this simple form does not, and the tile switch spills.  Off.
#ifndef ATTN8_PERSISTENT
#define ATTN8_PERSISTENT 0
#endif

// 1: in the steady state the copies of a stage are issued inside the pass, one piece behind each of a few
// MFMAs; 0: all of them right after the barrier.
#ifndef ATTN8_COPIES_IN_PASS
#define ATTN8_COPIES_IN_PASS 1
#endif

#ifdef ATTN8_TIMING
// Profiling builds only: cycle and wall-clock totals of the main loop of the first workgroups.
constexpr int DBG8_WGS = 1024, DBG8_SLOTS = 8;
__device__ unsigned long long attn8_dbg[DBG8_WGS * 8 * DBG8_SLOTS];
#endif

// (block scales 0, 0 select the plain, unscaled instruction)
__device__ __forceinline__ f32x16 mfma_fp8(i32x8 a, i32x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 0, 0, 0, 0, 0, 0);
}

__device__ __forceinline__ float xor32_max_fp8(float x) {
    // v_permlane32_swap swaps the upper 32 lanes of its first operand with the lower 32 lanes of its
    // second: afterwards a holds the lower half's value on every lane and b the upper half's.
    // (inline asm: the compiler folds the two results of the builtin into one when both inputs are
    // the same value; the s_nop covers the VALU-write -> permlane-read hazard)
    float a = x, b = x;
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
    return __builtin_fmaxf(a, b);
}

template <int OUT, int D, int BN, bool CAUSAL, bool PERSIST>
__global__ __launch_bounds__(512)
void attn_fwd_fp8_kernel(const uint8_t* __restrict__ q, const uint8_t* __restrict__ k, const uint8_t* __restrict__ v,
                         uint16_t* __restrict__ o, float* __restrict__ lse, int N, int nqt, int total,
                         float scale, float scale_log2e)
{
    typedef Elem<OUT> EO;
    constexpr int NW = 8, STAGES = ATTN8_STAGES;
    constexpr int AHEAD = STAGES - 2;           // iteration j issues the copies of stage j + AHEAD
    constexpr int BM = NW * 32;                 // query rows per workgroup
    constexpr int KB = BN / 32;                 // 32-key blocks per K/V tile
    constexpr int KC = BN / 64;                 // 64-key contraction steps of U
    constexpr int FK = D / 64;                  // contraction steps of T
    constexpr int DB = D / 32;                  // 32-wide feature blocks of O
    constexpr int CPR = D / 16;                 // 16-byte columns per row
    constexpr int RPB = 256 / D;                // rows per 256 bytes (one sweep over the LDS banks)
    constexpr int RPP = 1024 / D;               // rows per 1 KiB piece (one copy instruction)
    constexpr int TILE_BYTES = BN * D;          // one K or one V tile
    constexpr int STAGE_BYTES = 2 * TILE_BYTES;
    constexpr int CHUNKS = TILE_BYTES / 1024;   // pieces per tile
    constexpr int PPW = 2 * CHUNKS / NW;        // pieces (of K or V) a wave copies per stage
    static_assert(BN % 64 == 0 && (D == 64 || D == 128), "tile shape");
    static_assert((2 * CHUNKS) % NW == 0 && PPW >= 1, "a stage must split evenly over the eight waves");

    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const unsigned lds_base = (unsigned)(size_t)(LDS_AS void*)smem;

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    // ---- which (batch*head, query tile) this workgroup works on.  PERSIST (the causal launch): one workgroup per CU
    // walks the static serpentine schedule of tile_schedule.h round by round (the persistent, statically balanced
    // launch of the paper's Section 4.2: long and short query tiles are paired); otherwise one round.
    for (int round = 0;; ++round) {
    const int tile = __builtin_amdgcn_readfirstlane(tile_schedule(total, (int)gridDim.x, (int)blockIdx.x, round));
    if (tile < 0) break;
    // (the lane id is taken afresh in every round: everything derived from it then belongs to the round, and the
    // compiler does not hoist a dozen per-lane constants out of the loop and spill them)
    int lane;
    asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(lane));
    const int lr = lane & 31, g = lane >> 5;
    const int bh = __builtin_amdgcn_readfirstlane(tile / nqt);
    int qt = tile - bh * nqt;
    if (CAUSAL) qt = nqt - 1 - qt;              // long rows first
    const int q0 = qt * BM;
    const int wq0 = __builtin_amdgcn_readfirstlane(q0 + wave * 32);   // first query row of this wave
    const size_t head_off = (size_t)bh * N * D;
    const uint8_t* qh = q + head_off;
    const char* kh = uniform_ptr(reinterpret_cast<const char*>(k + head_off));
    const char* vh = uniform_ptr(reinterpret_cast<const char*>(v + head_off));
    int nt = (N + BN - 1) / BN;                 // K/V tiles the workgroup walks
    if (CAUSAL) nt = min(nt, (min(q0 + BM, N) - 1) / BN + 1);
    int nt_w = nt;                              // those this wave computes on (1 <= nt_w <= nt)
    if (CAUSAL) nt_w = min(nt, (wq0 + 31) / BN + 1);
    nt = __builtin_amdgcn_readfirstlane(nt);
    nt_w = __builtin_amdgcn_readfirstlane(nt_w);
    const int last_stage = max(AHEAD - 1, nt - 1);   // stages -2 .. last_stage are copied

    // ---- global -> LDS copies.  Stage s holds K tile s+2 and V tile s.  A tile is CHUNKS pieces of
    // 1 KiB (RPP whole rows each).  With an even number of pieces per wave every wave copies as many
    // K pieces as V pieces; with one piece per wave the first half of the waves copies K, the second V.
    // Lane L's 16 bytes land at piece + 16 L, i.e. row L / CPR of the piece, slot L % CPR; which
    // column of which global row it fetches follows from the layouts above.
    constexpr bool SPLIT = PPW % 2 == 0;
    unsigned piece_lane_off[PPW];               // per lane: byte offset of its 16 bytes inside the source tile
    int piece_row[PPW], piece_col[PPW];         // per lane: the tile-local source row and column of the same
    int piece_dst[PPW];                         // wave-uniform: byte offset of the piece inside the stage
    bool piece_is_v[PPW];                       // compile-time when SPLIT, else wave-uniform
    const char* piece_src[PPW];                 // wave-uniform: start of the tile that stage 0 takes (K tile 2 or V tile 0)
#pragma unroll
    for (int i = 0; i < PPW; ++i) {
        int pc;                                 // piece index inside its tile
        if (SPLIT) {
            piece_is_v[i] = i >= PPW / 2;
            pc = wave * (PPW / 2) + i % (PPW / 2 > 0 ? PPW / 2 : 1);
        } else {
            piece_is_v[i] = wave * PPW + i >= CHUNKS;
            pc = piece_is_v[i] ? wave * PPW + i - CHUNKS : wave * PPW + i;
        }
        const int p = pc * RPP + lane / CPR;    // LDS row of this lane's 16 bytes
        const int slot = lane % CPR;
        int row, col;
        if (piece_is_v[i]) {
            row = (p & ~12) | ((p & 4) << 1) | ((p & 8) >> 1);          // position p holds the key with bits 2, 3 swapped
            col = slot ^ (2 * ((p / RPB) % (CPR / 2)));
        } else {
            row = p;
            col = slot ^ ((p / RPB) % CPR);
        }
        piece_row[i] = row;
        piece_col[i] = col;
        piece_lane_off[i] = row * D + col * 16;
        piece_dst[i] = __builtin_amdgcn_readfirstlane((piece_is_v[i] ? TILE_BYTES : 0) + pc * 1024);
        piece_src[i] = uniform_ptr(piece_is_v[i] ? vh : kh + 2 * TILE_BYTES);
    }
    // Stage s lies wholly inside the sequence (K tile s+2 is its last one): scalar address arithmetic only.
    auto stage_inside = [&](int s) __attribute__((always_inline)) -> bool { return (s + 3) * BN <= N; };
    auto issue_inside = [&](int s) __attribute__((always_inline)) {
        const unsigned sbase = lds_base + ((s + 2 * STAGES) % STAGES) * STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < PPW; ++i)
            dma16(piece_src[i] + (size_t)s * TILE_BYTES, piece_lane_off[i], sbase + piece_dst[i]);
    };
    // any stage: rows clamped into the sequence (surplus rows are masked or never read)
    auto issue_stage = [&](int s) __attribute__((always_inline)) {
        const unsigned sbase = lds_base + ((s + 2 * STAGES) % STAGES) * STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < PPW; ++i) {
            const int t = piece_is_v[i] ? s : s + 2;                   // the tile this piece belongs to
            const int row = min(max(t * BN + piece_row[i], 0), N - 1);
            dma16(piece_is_v[i] ? vh : kh, (unsigned)(row * D + piece_col[i] * 16), sbase + piece_dst[i]);
        }
    };

    // ---- prologue: the whole ring in flight, then the Q fragments into registers.  The Q loads are ordinary
    // loads issued after the copies and waited for together with them: the compiler must know that their
    // destination registers are busy until the data is there (a load hidden in an asm statement lets it move or
    // reuse those registers while the load is still in flight).
#pragma unroll
    for (int s0 = -2; s0 < AHEAD; ++s0) issue_stage(s0);
    i32x8 Qf[FK];                               // B operand of T: query lane%32, features fk*64 + (lane/32)*32 .. +31
    {
        const int row = min(wq0 + lr, N - 1);
        const uint8_t* qr = qh + (size_t)row * D + g * 32;
#pragma unroll
        for (int fk = 0; fk < FK; ++fk) {
            const i32x4 lo = *reinterpret_cast<const i32x4*>(qr + fk * 64);
            const i32x4 hi = *reinterpret_cast<const i32x4*>(qr + fk * 64 + 16);
            Qf[fk] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        }
    }

    // A operand of the ones block: 1.0 in every byte, kept in registers for the whole kernel
    i32x8 ones;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        int w = 0x38383838;
        asm volatile("" : "+v"(w));
        ones[t] = w;
    }

    f32x16 O[DB], L, S[2][KB];                  // L: the ones block of the second contraction = row sums
    int pw[2][KB * 4] = {};                     // P of two consecutive tiles, four E4M3 values per word
    float m_run;

    // ---- per-lane LDS read offsets (the rest of every address is an immediate)
    // K fragment (A operand of T): key kb*32 + lane%32, features fk*64 + (lane/32)*32 .. +31 = columns
    // fk*4 + g*2 and the next one, each at its permuted slot.
    // All of a lane's fragment addresses inside a stage differ from ONE per-lane offset by an XOR with a
    // compile-time constant (the permuted 16-byte slot is column ^ f(row), and the column bits that vary
    // with the fragment are disjoint from those that vary with the lane), and a stage starts on a 1 KiB
    // boundary: (stage + offset) ^ constant is the address, one register per tile kind instead of one per
    // fragment column.
    const int k_lane0 = lr * D + (((g * 2) ^ ((lr / RPB) % CPR)) * 16);
    int v_lane0;
    {
        const int e = (lane & 15) >> 1, fh = (lane >> 4) & 1;
        const int p = g * 8 + e;
        v_lane0 = TILE_BYTES + p * D + ((fh ^ (2 * ((p / RPB) % (CPR / 2)))) * 16) + (lane & 1) * 8;
    }
    // (32-bit LDS addresses throughout: an XOR on a generic pointer would hide the address space from the compiler)
    auto lds_addr = [](const char* st, int off0, unsigned c) __attribute__((always_inline)) -> unsigned {
        return ((unsigned)(size_t)(LDS_AS const char*)st + (unsigned)off0) ^ c;
    };
    auto read_kf = [&](const char* st, int kb, int fk) __attribute__((always_inline)) -> i32x8 {
        const i32x4 lo = *(LDS_AS const i32x4*)(size_t)(lds_addr(st, k_lane0, (fk * 4) * 16) + kb * 32 * D);
        const i32x4 hi = *(LDS_AS const i32x4*)(size_t)(lds_addr(st, k_lane0, (fk * 4 + 1) * 16) + kb * 32 * D);
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    };
    auto read_vf = [&](const char* st, int kc, int db) __attribute__((always_inline)) -> i32x8 {
        const unsigned a = lds_addr(st, v_lane0, (db * 2) * 16) + kc * 64 * D;
        const i32x2 r0 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((LDS_AS i32x2*)(size_t)(a));
        const i32x2 r1 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((LDS_AS i32x2*)(size_t)(a + 16 * D));
        const i32x2 r2 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((LDS_AS i32x2*)(size_t)(a + 32 * D));
        const i32x2 r3 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((LDS_AS i32x2*)(size_t)(a + 48 * D));
        const i32x4 lo = __builtin_shufflevector(r0, r1, 0, 1, 2, 3);
        const i32x4 hi = __builtin_shufflevector(r2, r3, 0, 1, 2, 3);
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    };

    // ---- softmax state shared by the slices of one tile
    float sm_alpha = 1.f, sm_negmc = 0.f;
    bool sm_upd = false;
    // first slice: (mask,) row maximum, reference update, rescaling factor
    auto softmax_head = [&](auto par, auto masked, int j) __attribute__((always_inline)) {
        constexpr int P = decltype(par)::value;
        if (decltype(masked)::value) {
            const int kv0 = j * BN;
            const int qi = wq0 + lr;
            const int lim = CAUSAL ? min(qi, N - 1) : N - 1;   // last visible key
#pragma unroll
            for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int key = kv0 + kb * 32 + (i >> 2) * 8 + g * 4 + (i & 3);
                    if (key > lim) S[P][kb][i] = -__builtin_inff();
                }
        }
        float mx = S[P][0][0];
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int i = 0; i < 16; ++i) mx = __builtin_fmaxf(mx, S[P][kb][i]);
        mx = xor32_max_fp8(mx);
        const float m_old = m_run;
        const float m_new = __builtin_fmaxf(m_old, mx);
        sm_upd = (m_new - m_old) * scale_log2e > RESCALE_LOG2_FP8;
        const float m_use = sm_upd ? m_new : m_old;
        sm_alpha = __builtin_amdgcn_exp2f((m_old - m_use) * scale_log2e);
        sm_negmc = -m_use * scale_log2e;
        m_run = m_use;
    };
    // slice g4 of KB*4: four scores -> one word of E4M3 probabilities
    auto softmax_group = [&](auto par, int g4) __attribute__((always_inline)) {
        constexpr int P = decltype(par)::value;
        const int kb = g4 / 4, t = g4 % 4;
        const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(S[P][kb][4 * t + 0], scale_log2e, sm_negmc));
        const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(S[P][kb][4 * t + 1], scale_log2e, sm_negmc));
        const float p2 = __builtin_amdgcn_exp2f(__builtin_fmaf(S[P][kb][4 * t + 2], scale_log2e, sm_negmc));
        const float p3 = __builtin_amdgcn_exp2f(__builtin_fmaf(S[P][kb][4 * t + 3], scale_log2e, sm_negmc));
        // (the first conversion fills the low half of the word and keeps the rest, the second fills the
        // high half: starting from the word's previous content saves clearing a register)
        int w = __builtin_amdgcn_cvt_pk_fp8_f32(p0, p1, pw[P][kb * 4 + t], false);
        w = __builtin_amdgcn_cvt_pk_fp8_f32(p2, p3, w, true);
        // (pins the slice where it is written: the word is only used by the next pass, and the
        // compiler would otherwise sink the whole slice down to that use)
        asm volatile("" : "+v"(w));
        pw[P][kb * 4 + t] = w;
    };
    // after the U of the previous tile: move O and L to the new reference (rare after the first tiles)
    auto softmax_rescale = [&]() __attribute__((always_inline)) {
        if (__builtin_amdgcn_ballot_w64(sm_upd) != 0) {
#pragma unroll
            for (int db = 0; db < DB; ++db) O[db] = O[db] * sm_alpha;
            L = L * sm_alpha;
        }
    };

    // ---- one pass over a stage: the MFMAs of U (the ones block and O^T += V^T P^T, P of parity
    // PAR^1) and/or T (S^T of parity PAR^1 = K Q^T), LDS fragments requested FWIN MFMAs ahead, and,
    // between the MFMAs, the softmax of the scores of parity PAR (tile j): the row maximum after the
    // first MFMA, then one slice of scores after each of the others.  The scheduling barriers keep
    // that order.  (Measured: the row maximum before the first MFMA, the ones block first, or the
    // maximum in four independent chains each change the time by 1-3 % the wrong way.)
    // `copies`: the pass also issues the copies of stage j + AHEAD (known to lie wholly inside the
    // sequence), one piece after each of a few MFMAs: the wave is held while a copy instruction hands
    // its addresses to the memory pipeline, and behind an MFMA of its own that time costs nothing.
    auto pass = [&](auto do_u, auto do_t, auto do_c, auto copies, auto par, const char* st, int j) __attribute__((always_inline)) {
        constexpr int P = decltype(par)::value;
        constexpr bool COPIES = decltype(copies)::value;
        constexpr bool C = decltype(do_c)::value;
        constexpr int UB = DB + 1;                                      // per 64 keys: DB feature blocks, then the ones block
        constexpr int NU = decltype(do_u)::value ? KC * UB : 0;
        constexpr int NT = decltype(do_t)::value ? KB * FK : 0;
        constexpr int NF = NU + NT;
        constexpr int FWIN = ATTN8_FWIN < NF ? ATTN8_FWIN : NF;
        constexpr int NG = KB * 4;                                      // softmax slices after the head
        constexpr bool IL = C && ATTN8_INTERLEAVE && NF >= 2;
        i32x8 fr[NF > 0 ? NF : 1];
        auto fetch = [&](int f) __attribute__((always_inline)) {
            if (f < NU) {
                const int kc = f / UB, db = (f % UB) == DB ? -1 : f % UB;
                if (db >= 0) fr[f] = read_vf(st, kc, db);
                else fr[f] = ones;
            } else {
                fr[f] = read_kf(st, (f - NU) % KB, (f - NU) / KB);
            }
        };
        auto run_mfma = [&](int f) __attribute__((always_inline)) {
            if (f < NU) {
                const int kc = f / UB, db = (f % UB) == DB ? -1 : f % UB;
                i32x8 p;
#pragma unroll
                for (int t = 0; t < 8; ++t) p[t] = pw[P ^ 1][kc * 8 + t];
                if (db >= 0) O[db] = mfma_fp8(fr[f], p, O[db]);
                else L = mfma_fp8(fr[f], p, L);
            } else {
                const int kb = (f - NU) % KB, fk = (f - NU) / KB;
                S[P ^ 1][kb] = mfma_fp8(fr[f], Qf[fk], fk == 0 ? f32x16(0.f) : S[P ^ 1][kb]);
            }
        };
#pragma unroll
        for (int f = 0; f < FWIN; ++f) fetch(f);
#pragma unroll
        for (int f = 0; f < NF; ++f) {
            if (f + FWIN < NF) fetch(f + FWIN);
            run_mfma(f);
            __builtin_amdgcn_sched_barrier(0);
            if (COPIES) {
                // pieces after MFMAs 1, 3, 5, ... (the first MFMA is followed by the row maximum)
#pragma unroll
                for (int i = 0; i < PPW; ++i)
                    if (f == 1 + 2 * i || (1 + 2 * i >= NF && f == NF - 1 && i >= (NF - 1) / 2)) {
                        const int s = j + AHEAD;
                        dma16(piece_src[i] + (size_t)s * TILE_BYTES, piece_lane_off[i],
                              lds_base + ((s + 2 * STAGES) % STAGES) * STAGE_BYTES + piece_dst[i]);
                    }
                __builtin_amdgcn_sched_barrier(0);
            }
            if (IL) {
                if (f == 0) {
                    softmax_head(par, std::false_type{}, j);
                } else {
                    // slices (f-1)*NG/(NF-1) .. f*NG/(NF-1) - 1 (rounded up), so that the last MFMA takes the last slice
#pragma unroll
                    for (int s = ((f - 1) * NG + NF - 2) / (NF - 1); s < (f * NG + NF - 2) / (NF - 1); ++s) softmax_group(par, s);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        if (C && !IL) {
            softmax_head(par, std::false_type{}, j);
#pragma unroll
            for (int s = 0; s < NG; ++s) softmax_group(par, s);
        }
        if (C) softmax_rescale();
    };

    // Barrier j: every wave's share of the stages up to j has landed (the copies of the stages after
    // it, at most AHEAD - 1 of them, may still be in flight) and nobody reads stage j-2 any more, so
    // that slot takes the copies of stage j + AHEAD.
    auto step = [&](int j, bool with_copies = true) __attribute__((always_inline)) {
        const int n_out = min(j + AHEAD - 1, last_stage) - j;           // stages that may stay in flight
        if (n_out >= AHEAD - 1) wait_vmcnt<(AHEAD - 1) * PPW>();
        else if (n_out == 4 && AHEAD > 5) wait_vmcnt<4 * PPW>();
        else if (n_out == 3 && AHEAD > 4) wait_vmcnt<3 * PPW>();
        else if (n_out == 2 && AHEAD > 3) wait_vmcnt<2 * PPW>();
        else if (n_out == 1 && AHEAD > 2) wait_vmcnt<1 * PPW>();
        else wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();
        const int s = j + AHEAD;
        if (with_copies && s <= last_stage) {
            if (stage_inside(s)) issue_inside(s); else issue_stage(s);
        }
    };
    auto stage_ptr = [&](int s) __attribute__((always_inline)) -> const char* { return smem + ((s + 2 * STAGES) % STAGES) * STAGE_BYTES; };

    // Use the Q fragments once here: the compiler then waits for their loads now (its vmcnt(0) also covers the
    // copies issued before them) instead of inside the first pass.  (Word by word: the host pass of the compiler
    // silently drops a kernel whose inline asm takes a 256-bit operand.)
#pragma unroll
    for (int fk = 0; fk < FK; ++fk)
#pragma unroll
        for (int t = 0; t < 8; ++t) asm volatile("" :: "v"(Qf[fk][t]));
    wait_vmcnt<0>();
    m_run = -__builtin_inff();
    L = f32x16(0.f);
#pragma unroll
    for (int db = 0; db < DB; ++db) O[db] = f32x16(0.f);
    __builtin_amdgcn_s_barrier();               // stages -2 .. 0 are complete for every wave
#ifdef ATTN8_TIMING
    const unsigned long long rt0 = __builtin_amdgcn_s_memrealtime(), ct0 = __builtin_readcyclecounter();
#endif

    constexpr std::integral_constant<int, 0> P0{};
    constexpr std::integral_constant<int, 1> P1{};
    constexpr std::true_type Y{};
    constexpr std::false_type NO{};

    // Iteration j of a wave (after barrier j; it reads stage j-1 = K tile j+1, V tile j-1, and at its
    // end the first fragments of stage j):
    //   j <= nt_w - 2   MFMAs of U_{j-1} and T_{j+1}, softmax C_j in between (no tile before the last needs a mask)
    //   j == nt_w - 1   U_{j-1}, then C_j with the mask (diagonal or ragged end), then U_j (stage j is visible)
    //   j >= nt_w       nothing: the wave only keeps copying its share for the others
    pass(NO, Y, NO, NO, P1, stage_ptr(-2), 0);                          // T_0 into the scores of parity 0
    int j = 0;
    if (nt_w >= 2) {
        step(0);
        pass(NO, Y, Y, NO, P0, stage_ptr(-1), 0);                       // T_1 and C_0
        j = 1;
        // first the iterations whose copies (stage j + AHEAD) lie wholly inside the sequence: the pass issues them
        const int j_in = min(nt_w - 2, N / BN - AHEAD - 3);
        if (ATTN8_COPIES_IN_PASS && j + 1 <= j_in) {
            do {                                // bottom-tested: the accumulators are updated in place
                step(j, false);
                pass(Y, Y, Y, Y, P1, stage_ptr(j - 1), j);
                step(j + 1, false);
                pass(Y, Y, Y, Y, P0, stage_ptr(j), j + 1);
                j += 2;
            } while (j + 1 <= j_in);
        }
        if (j + 1 <= nt_w - 2) {
            do {
                step(j);
                pass(Y, Y, Y, NO, P1, stage_ptr(j - 1), j);
                step(j + 1);
                pass(Y, Y, Y, NO, P0, stage_ptr(j), j + 1);
                j += 2;
            } while (j + 1 <= nt_w - 2);
        }
        if (j <= nt_w - 2) {
            step(j);
            pass(Y, Y, Y, NO, P1, stage_ptr(j - 1), j);
            ++j;
        }
    }
    // j == nt_w - 1: the last tile this wave computes on
    auto tail = [&](auto par, auto parx) __attribute__((always_inline)) {
        step(j);
        if (j >= 1) pass(Y, NO, NO, NO, par, stage_ptr(j - 1), j);      // U_{j-1}
        softmax_head(par, Y, j);
        __builtin_amdgcn_sched_barrier(0);      // (slice by slice: scheduled as one block this part spills more registers)
#pragma unroll
        for (int s = 0; s < KB * 4; ++s) {
            softmax_group(par, s);
            __builtin_amdgcn_sched_barrier(0);
        }
        softmax_rescale();
        pass(Y, NO, NO, NO, parx, stage_ptr(j), j + 1);                 // U_j
    };
    if (j & 1) tail(P1, P0); else tail(P0, P1);
    for (++j; j < nt; ++j) step(j);                               // idle tail of a causal wave
    wait_vmcnt<0>();

    // ---- epilogue: normalise, write O (16-bit) and LSE (natural log)
    {
        uint16_t* oh = o + head_off;
        float* lh = lse + (size_t)bh * N;
        const float l_tot = L[0];               // every element of the ones block holds the row sum
        const float inv = 1.0f / l_tot;
        const int row = wq0 + lr;
        if (row < N) {
            if (g == 0) lh[row] = m_run * scale + __builtin_logf(l_tot);
            uint16_t* orow = oh + (size_t)row * D;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) {
                    u32x2 w;
                    w[0] = EO::pack2(O[db][i4 * 4 + 0] * inv, O[db][i4 * 4 + 1] * inv);
                    w[1] = EO::pack2(O[db][i4 * 4 + 2] * inv, O[db][i4 * 4 + 3] * inv);
                    *reinterpret_cast<u32x2*>(orow + db * 32 + i4 * 8 + g * 4) = w;
                }
        }
    }
    if (!PERSIST) break;
    __builtin_amdgcn_s_barrier();               // every wave is done reading the ring before the next tile's copies go out
    }   // rounds
#ifdef ATTN8_TIMING
    if (blockIdx.x < DBG8_WGS && lane == 0) {
        unsigned long long* d = attn8_dbg + (blockIdx.x * 8 + wave) * DBG8_SLOTS;
        d[5] = nt;
        d[6] = __builtin_amdgcn_s_memrealtime() - rt0;   // 100 MHz ticks
        d[7] = __builtin_readcyclecounter() - ct0;
    }
#endif
}

#ifdef ATTN8_TIMING
}  // namespace
extern "C" int attn8_dbg_read(unsigned long long* host, int n)
{
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(attn8_dbg), sizeof(unsigned long long) * n);
}
namespace {
#endif

template <int OUT, int D, int BN, bool CAUSAL, bool PERSIST>
int launch_fp8(const AttnLaunchArgs& a)
{
    constexpr int BM = 256;
    constexpr int smem = ATTN8_STAGES * 2 * BN * D;
    auto kern = attn_fwd_fp8_kernel<OUT, D, BN, CAUSAL, PERSIST>;
    static PerDeviceOnce once;                  // the attribute belongs to the (kernel, device) pair
    const int dev = once.prepare(reinterpret_cast<const void*>(kern), smem);
    if (dev < 0) return -1;
    const int nqt = (a.N + BM - 1) / BM;
    const long long total = (long long)nqt * a.B * a.H;
    // Persistent launch: one workgroup per CU (eight waves at two per SIMD fill it), each walking its share of the schedule.
    long long grid = total;
    if (PERSIST) {
        const int cus = once.compute_units(dev);
        if (cus < 8) return -1;
        if (grid > cus) grid = cus;
    }
    const float log2e = 1.4426950408889634f;
    const uint8_t* q = (const uint8_t*)a.q;
    const uint8_t* k = (const uint8_t*)a.k;
    const uint8_t* v = (const uint8_t*)a.v;
    uint16_t* o = (uint16_t*)a.o;
    float* lse = a.lse;
    int N = a.N, nqt_arg = nqt, total_arg = (int)total;
    float scale = a.scale, scale_log2e = a.scale * log2e;
    void* args[] = {&q, &k, &v, &o, &lse, &N, &nqt_arg, &total_arg, &scale, &scale_log2e};
    const hipError_t e = hipLaunchKernel(reinterpret_cast<const void*>(kern), dim3((unsigned)grid), dim3(512),
                                         args, smem, (hipStream_t)a.stream);
    return e == hipSuccess ? 0 : -1;
}

template <int OUT, int D>
int launch_fp8_d(const AttnLaunchArgs& a)
{
    constexpr int BN = D == 128 ? ATTN8_CFG_BN_D128 : ATTN8_CFG_BN_D64;
    if (a.causal) return ATTN8_PERSISTENT ? launch_fp8<OUT, D, BN, true, true>(a) : launch_fp8<OUT, D, BN, true, false>(a);
    return launch_fp8<OUT, D, BN, false, false>(a);
}

}  // namespace

// a.dtype is the element type of O here (0 = fp16, 1 = bf16); Q, K, V are E4M3.
int attn_fp8_launch(const AttnLaunchArgs& a)
{
    if (a.dtype == 0) return a.d == 128 ? launch_fp8_d<0, 128>(a) : launch_fp8_d<0, 64>(a);
    return a.d == 128 ? launch_fp8_d<1, 128>(a) : launch_fp8_d<1, 64>(a);
}

int attn_fp8_launch_tile_param(int d, int which)
{
    if (d != 64 && d != 128) return -1;
    switch (which) {
        case 0: return 256;
        case 1: return d == 128 ? ATTN8_CFG_BN_D128 : ATTN8_CFG_BN_D64;
        case 2: return ATTN8_STAGES;
        case 3: return 512;
        default: return -1;
    }
}
