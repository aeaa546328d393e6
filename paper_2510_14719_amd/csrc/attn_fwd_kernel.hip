// Fused attention forward for gfx950 (MI355X): O = softmax(scale * Q K^T [+ causal mask]) V and
// per-row log-sum-exp, in one kernel with a streaming softmax.
//
// The three stages of one key/value tile follow the paper's Section 3.4.2: T = Q K^T on the matrix
// cores, C = softmax on the vector ALU, U = P V on the matrix cores.  The paper's Hopper design
// (a producer warp feeding consumer warp groups through asynchronous references, Section 3.2-3.3)
// is replaced by what gfx950 offers: every wave of a workgroup issues its share of the global -> LDS
// copies of the K/V tile two tiles ahead (direct-to-LDS loads, no register staging), the LDS holds a
// ring of STAGES tiles (the counterpart of an aref ring of depth D, Section 3.3.2), and one
// s_waitcnt + s_barrier per tile plays the role of the full/empty credits: a stage is overwritten
// only after every wave has passed the barrier that follows its last read of it.
//
// Register layout.  The scores are computed transposed, S^T = K Q^T, with the 32x32x16 MFMA: the
// K tile is the A operand (32 keys x 16 features), Q^T the B operand.  A lane then owns ONE query
// (column lane%32 of the result) and 16 of the 32 keys of a block; the other 16 keys of that query
// sit in lane^32.  Row maximum and row sum are 15 in-lane operations plus one lane<->lane+32
// exchange, and the probabilities are already laid out as the B operand of the second contraction
// O^T = V^T P^T.  V^T fragments come from the LDS through the transposing 64-bit read of gfx950.

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "attn_launch.h"

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

#define LDS_AS __attribute__((address_space(3)))

// The softmax reference moves only when a row maximum grew by more than this many powers of two.
constexpr float RESCALE_LOG2 = 8.0f;

// Tuning knobs of the hand-interleaved pipeline (see tile_step).
#ifndef ATTN_KWIN
#define ATTN_KWIN 3
#endif
#ifndef ATTN_VWIN
#define ATTN_VWIN 3
#endif

// Element-type traits: MFMA flavour and fp32 -> 16-bit conversion (round to nearest even).
template <int DTYPE> struct Elem;
template <> struct Elem<0> {  // IEEE binary16
    typedef _Float16 v8 __attribute__((ext_vector_type(8)));
    typedef _Float16 v2 __attribute__((ext_vector_type(2)));
    static __device__ __forceinline__ f32x16 mfma(s16x8 a, s16x8 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8, a), __builtin_bit_cast(v8, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ unsigned pack2(float lo, float hi) {
        f32x2 x = {lo, hi};
        return __builtin_bit_cast(unsigned, __builtin_convertvector(x, v2));
    }
};
template <> struct Elem<1> {  // bfloat16
    typedef __bf16 v8 __attribute__((ext_vector_type(8)));
    typedef __bf16 v2 __attribute__((ext_vector_type(2)));
    static __device__ __forceinline__ f32x16 mfma(s16x8 a, s16x8 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8, a), __builtin_bit_cast(v8, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ unsigned pack2(float lo, float hi) {
        f32x2 x = {lo, hi};
        return __builtin_bit_cast(unsigned, __builtin_convertvector(x, v2));
    }
};

// 16 bytes per lane from global memory straight into the LDS: lane L's bytes land at
// lds_addr + 16*L.  The compiler is not told about the transfer (it would otherwise wait for ALL
// outstanding loads before every LDS read); completion is tracked by hand with s_waitcnt vmcnt.
__device__ __forceinline__ void dma16(const void* gbase, unsigned voff, unsigned lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_addr), "v"(voff), "s"(gbase) : "memory");
}

template <int N> __device__ __forceinline__ void wait_vmcnt() {
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

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

// Workgroups are handed to the 8 XCDs round-robin; give every XCD a contiguous range of logical
// tiles so that the workgroups resident on one XCD stream the same head's K/V through its L2.
__device__ __forceinline__ int xcd_remap(int id, int total) {
    constexpr int XCDS = 8;
    const int q = total / XCDS, r = total % XCDS;
    const int x = id % XCDS, slot = id / XCDS;
    return x * q + (x < r ? x : r) + slot;
}

template <int DTYPE, int D, int NW, int MB, int BN, int STAGES, bool CAUSAL>
__global__ __launch_bounds__(NW * 64)
void attn_fwd_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
                     uint16_t* __restrict__ o, float* __restrict__ lse, int N, int nqt, int total,
                     float scale, float scale_log2e)
{
    typedef Elem<DTYPE> E;
    constexpr int BM = NW * MB * 32;            // query rows per workgroup
    constexpr int KB = BN / 32;                 // 32-key blocks ("halves") per K/V tile
    constexpr int KK = D / 16;                  // contraction steps of Q K^T
    constexpr int DB = D / 32;                  // 32-wide feature blocks of O
    constexpr int ROW_BYTES = D * 2;
    constexpr int TILE_BYTES = BN * ROW_BYTES;  // one K or one V tile
    constexpr int STAGE_BYTES = 2 * TILE_BYTES;
    constexpr int RB = BN / 16;                 // 16-row blocks per tile
    constexpr int CHUNKS = TILE_BYTES / 1024;   // 1 KiB wave-transfers per tile
    constexpr int CPW = CHUNKS / NW;            // ... per wave
    static_assert(CHUNKS % NW == 0, "tile must split evenly over the waves");
    static_assert(STAGES == 4, "the ring protocol below keeps tiles j..j+3 in four stages");
    static_assert(KB == 2, "a tile is processed as two 32-key halves");

    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const unsigned lds_base = (unsigned)(size_t)(LDS_AS void*)smem;

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform, kept in an SGPR
    const int lane = threadIdx.x & 63;
    const int lr = lane & 31, g = lane >> 5;

    // ---- which (batch*head, query tile) this workgroup owns
    const int logical = xcd_remap(blockIdx.x, total);
    const int bh = logical / nqt;
    int qt = logical - bh * nqt;
    if (CAUSAL) qt = nqt - 1 - qt;              // long rows first
    const int q0 = qt * BM;
    const int wq0 = q0 + wave * (MB * 32);      // first query row of this wave

    const size_t head_off = (size_t)bh * N * D;
    const uint16_t* qh = q + head_off;
    const char* kh = reinterpret_cast<const char*>(k + head_off);
    const char* vh = reinterpret_cast<const char*>(v + head_off);

    // ---- number of K/V tiles the workgroup walks, and of 32-key halves this wave computes on
    int nt = (N + BN - 1) / BN;
    if (CAUSAL) {
        const int last_q = min(q0 + BM, N) - 1;
        nt = min(nt, last_q / BN + 1);
    }
    int nh_w = min(2 * nt, (N + 31) / 32);                              // halves that hold a real key
    if (CAUSAL) nh_w = min(nh_w, (wq0 + MB * 32 - 1) / 32 + 1);         // ... and one this wave's rows can see

    // ---- global -> LDS copies.  A wave moves CPW 1 KiB pieces of K and of V per tile.
    // K tile in LDS: [feature group of 32][16-row block][16-byte column of the group (4)][row (16)][16 B]
    // V tile in LDS: [feature group of 32][row (BN)][64 B]
    // Lane L of a K piece fetches row L%16, column L/16 of the piece's (16 rows x 64 B) source block; of
    // a V piece row L/4, column L%4.  Inside the sequence the per-lane offset is a constant and the
    // tile/piece offset is added to the scalar base; the clamped form serves the tile that overruns N.
    const unsigned k_lane_off = (lane & 15) * ROW_BYTES + (lane >> 4) * 16;
    const unsigned v_lane_off = (lane >> 2) * ROW_BYTES + (lane & 3) * 16;
    auto issue_tile = [&](int t, int stage) {
        const int kv0 = t * BN;
        const unsigned sbase = lds_base + stage * STAGE_BYTES;
        if (kv0 + BN <= N) {
#pragma unroll
            for (int i = 0; i < CPW; ++i) {
                const int wc = wave * CPW + i, fg = wc / RB, rb = wc % RB;
                const size_t off = (size_t)(kv0 + rb * 16) * ROW_BYTES + fg * 64;
                dma16(kh + off, k_lane_off, sbase + wc * 1024);
            }
#pragma unroll
            for (int i = 0; i < CPW; ++i) {
                const int wc = wave * CPW + i, fg = wc / RB, rb = wc % RB;
                const size_t off = (size_t)(kv0 + rb * 16) * ROW_BYTES + fg * 64;
                dma16(vh + off, v_lane_off, sbase + TILE_BYTES + wc * 1024);
            }
        } else {
#pragma unroll
            for (int i = 0; i < CPW; ++i) {
                const int wc = wave * CPW + i, fg = wc / RB, rb = wc % RB;
                const int row = min(kv0 + rb * 16 + (lane & 15), N - 1);
                dma16(kh, (unsigned)(row * ROW_BYTES + fg * 64 + (lane >> 4) * 16), sbase + wc * 1024);
            }
#pragma unroll
            for (int i = 0; i < CPW; ++i) {
                const int wc = wave * CPW + i, fg = wc / RB, rb = wc % RB;
                const int row = min(kv0 + rb * 16 + (lane >> 2), N - 1);
                dma16(vh, (unsigned)(row * ROW_BYTES + fg * 64 + (lane & 3) * 16), sbase + TILE_BYTES + wc * 1024);
            }
        }
    };

    // ---- prologue: up to three tiles in flight, Q fragments into registers
    issue_tile(0, 0);
    if (nt > 1) issue_tile(1, 1);
    if (nt > 2) issue_tile(2, 2);

    s16x8 Qf[MB][KK];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const int row = min(wq0 + mb * 32 + lr, N - 1);
        const uint16_t* qr = qh + (size_t)row * D;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk)
            Qf[mb][kk] = *reinterpret_cast<const s16x8*>(qr + (kk * 2 + g) * 8);
    }
    // Use the Q fragments once here: the compiler then waits for their loads before the loop instead
    // of inside it, where its vmcnt(0) would also wait for the K/V copies issued a moment earlier.
    // (The Q loads were issued after the tile copies, so this wait also covers tiles 0..2.)
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) asm volatile("" :: "v"(Qf[mb][kk]));

    f32x16 O[MB][DB];
    float m_run[MB], l_run[MB], alpha[MB], neg_mc[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        m_run[mb] = -__builtin_inff();
        l_run[mb] = 0.f;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) O[mb][db][i] = 0.f;
    }
    bool any_upd = false;

    // per-lane LDS read offsets (the rest of every address is an immediate)
    const int k_lane = (lr >> 4) * 1024 + g * 256 + (lr & 15) * 16;
    const int v_lane = TILE_BYTES + (4 * g + ((lane & 15) >> 2)) * 64 + ((lane >> 4) & 1) * 32 + (lane & 3) * 8;

    // K fragment (A operand of T): keys kb*32 + lane%32, features (kk*2 + lane/32)*8 .. +7
    auto read_kf = [&](const char* sk, int kb, int kk) -> s16x8 {
        return *reinterpret_cast<const s16x8*>(sk + ((kk >> 1) * RB + kb * 2) * 1024 + (kk & 1) * 512);
    };
    // V^T fragment (A operand of U): features db*32 + lane%32, the 8 keys of half kb that the P
    // operand of MFMA ks holds in this lane group, fetched with the transposing LDS read
    auto read_vf = [&](const char* sv, int kb, int ks, int db) -> s16x8 {
        const char* a = sv + db * (BN * 64) + (kb * 32 + ks * 16) * 64;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(a));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(a + 8 * 64));
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    };

    // mask of one half's scores: keys past the end of the sequence, and keys after the query when causal
    auto mask_half = [&](f32x16 (&S)[MB], int key0) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            const int qi = wq0 + mb * 32 + lr;
            const int lim = CAUSAL ? min(qi, N - 1) : N - 1;   // last visible key
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int key = key0 + (i >> 2) * 8 + g * 4 + (i & 3);
                if (key > lim) S[mb][i] = -__builtin_inff();
            }
        }
    };
    auto half_needs_mask = [&](int h) -> bool {
        const int key_last = h * 32 + 31;
        return key_last > N - 1 || (CAUSAL && key_last > wq0);
    };

    // First part of C for one half: from its row maxima `mx`, the new softmax reference.  The running
    // reference m only moves when a row maximum grew by more than 2^RESCALE_LOG2 (the probabilities
    // then stay below that factor), so the rescaling of O is rare after the first tiles.
    auto new_reference = [&](const float (&mx)[MB]) {
        bool upd_any = false;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            const float mxa = xor32_max(mx[mb]);
            const float m_old = m_run[mb];
            const float m_new = __builtin_fmaxf(m_old, mxa);
            const bool upd = (m_new - m_old) * scale_log2e > RESCALE_LOG2;
            const float m_use = upd ? m_new : m_old;
            upd_any |= upd;
            alpha[mb] = __builtin_amdgcn_exp2f((m_old - m_use) * scale_log2e);
            neg_mc[mb] = -m_use * scale_log2e;
            m_run[mb] = m_use;
        }
        any_upd = __builtin_amdgcn_ballot_w64(upd_any) != 0;
    };

    // ---- one step of the coarse-grained pipeline (Algorithm 1 of the paper, in its dependency-correct
    // order) on a 32-key half h of the sequence.  On entry S holds the half's masked scores and
    // new_reference() has been run on them.
    //   matrix cores: T_{h+1} = K_{h+1} Q^T                then U_h = V_h^T P_h^T
    //   vector ALU:   exponentials, row sums, P of half h   then row maxima / reference of half h+1
    // The two streams are interleaved by hand, one MFMA per chunk of vector work, and a scheduling
    // barrier after every chunk keeps the compiler from regrouping them: an MFMA executes for 32
    // cycles after it is issued and the vector instructions behind it run in its shadow.
    // sk: K tile holding half h+1 (+ k_lane), sv: V tile holding half h (+ v_lane).
    auto half_step = [&](auto maskn_c, auto next_c, f32x16 (&S)[MB], f32x16 (&Sn)[MB], int h, const char* sk, const char* sv) {
        constexpr bool MASKN = decltype(maskn_c)::value;
        constexpr bool NEXT = decltype(next_c)::value;
        constexpr int KWIN = ATTN_KWIN < KK ? ATTN_KWIN : KK;          // K fragments requested ahead of their MFMA
        constexpr int NVF = 2 * DB;                                    // V^T fragments (= MFMAs of U per query block)
        constexpr int VWIN = ATTN_VWIN < NVF ? ATTN_VWIN : NVF;        // V^T fragments requested ahead
        constexpr int EPC = 16 / KK;                                   // scores handled next to each MFMA of T
        constexpr int MPC = 16 / NVF;                                  // maxima handled next to each MFMA of U
        static_assert(EPC >= 2 && EPC % 2 == 0 && MPC >= 1 && VWIN <= KK, "chunking of the vector work");
        const int kbn = (h + 1) & 1, kbc = h & 1;                      // position of the halves inside their tiles

        if (any_upd) {
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int i = 0; i < 16; ++i) O[mb][db][i] *= alpha[mb];
        }

        // ---- phase 1: T_{h+1} under the exponentials of half h
        s16x8 kf[KK], vf[NVF];
        unsigned pw[MB][8];
        float sum[MB];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) sum[mb] = 0.f;
        if (NEXT) {
#pragma unroll
            for (int i = 0; i < KWIN; ++i) kf[i] = read_kf(sk, kbn, i);
        }
#pragma unroll
        for (int i = 0; i < KK; ++i) {
            if (NEXT) {
                if (i + KWIN < KK) kf[i + KWIN] = read_kf(sk, kbn, i + KWIN);
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    if (i == 0) {
                        f32x16 z;
#pragma unroll
                        for (int e = 0; e < 16; ++e) z[e] = 0.f;
                        Sn[mb] = E::mfma(kf[i], Qf[mb][i], z);
                    } else {
                        Sn[mb] = E::mfma(kf[i], Qf[mb][i], Sn[mb]);
                    }
                }
            }
            if (i + VWIN >= KK) {                               // the first V^T fragments, late in the phase
                const int f = i + VWIN - KK;
                vf[f] = read_vf(sv, kbc, f / DB, f % DB);
            }
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                float pe[EPC];
#pragma unroll
                for (int e = 0; e < EPC; ++e) {
                    pe[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(S[mb][EPC * i + e], scale_log2e, neg_mc[mb]));
                    sum[mb] += pe[e];
                }
#pragma unroll
                for (int e = 0; e < EPC; e += 2) pw[mb][(EPC * i + e) / 2] = E::pack2(pe[e], pe[e + 1]);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) l_run[mb] = l_run[mb] * alpha[mb] + sum[mb];

        // ---- phase 2: U_h under the row maxima of half h+1
        if (NEXT && MASKN) mask_half(Sn, (h + 1) * 32);
        float mx[MB];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) mx[mb] = -__builtin_inff();
#pragma unroll
        for (int f = 0; f < NVF; ++f) {
            if (f + VWIN < NVF) vf[f + VWIN] = read_vf(sv, kbc, (f + VWIN) / DB, (f + VWIN) % DB);
            const int ks = f / DB, db = f % DB;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                u32x4 w;
#pragma unroll
                for (int t = 0; t < 4; ++t) w[t] = pw[mb][ks * 4 + t];
                O[mb][db] = E::mfma(vf[f], __builtin_bit_cast(s16x8, w), O[mb][db]);
            }
            if (NEXT) {
#pragma unroll
                for (int e = f * MPC; e < (f + 1) * MPC; ++e)
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb) mx[mb] = __builtin_fmaxf(mx[mb], Sn[mb][e]);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        if (NEXT) new_reference(mx);
    };

    auto run_half = [&](f32x16 (&S)[MB], f32x16 (&Sn)[MB], int h, const char* sk, const char* sv) {
        if (h >= nh_w) return;
        if (h + 1 < nh_w) {
            if (half_needs_mask(h + 1)) half_step(std::true_type{}, std::true_type{}, S, Sn, h, sk, sv);
            else half_step(std::false_type{}, std::true_type{}, S, Sn, h, sk, sv);
        } else {
            half_step(std::false_type{}, std::false_type{}, S, Sn, h, sk, sv);
        }
    };

    // ---- T_0 and its reference, not overlapped with anything
    f32x16 Sa[MB], Sb[MB];
    __builtin_amdgcn_s_barrier();      // every wave's share of tile 0 is in the LDS
    {
        const char* sk = smem + k_lane;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            const s16x8 kf = read_kf(sk, 0, kk);
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                if (kk == 0) {
                    f32x16 z;
#pragma unroll
                    for (int e = 0; e < 16; ++e) z[e] = 0.f;
                    Sa[mb] = E::mfma(kf, Qf[mb][kk], z);
                } else {
                    Sa[mb] = E::mfma(kf, Qf[mb][kk], Sa[mb]);
                }
            }
        }
        if (half_needs_mask(0)) mask_half(Sa, 0);
        float mx[MB];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            mx[mb] = Sa[mb][0];
#pragma unroll
            for (int e = 1; e < 16; ++e) mx[mb] = __builtin_fmaxf(mx[mb], Sa[mb][e]);
        }
        new_reference(mx);
        any_upd = false;               // O is still zero: nothing to rescale
    }

    // ---- main loop over the K/V tiles; each tile is two half steps, so Sa/Sb swap roles twice per tile.
    // sync(j): tile j+1 (read by the second half step) has landed once at most tile j+2's copies are
    // outstanding; the barrier extends that to every wave's share and tells that tile j-1 is no
    // longer read, so its stage can take tile j+3.
    int stage = 0;
    auto sync_and_prefetch = [&](int j) {
        if (j + 2 < nt) wait_vmcnt<2 * CPW>(); else wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();
        if (j + 3 < nt) issue_tile(j + 3, (stage + 3) % STAGES);
    };

    // Halves before `h_plain_end` need no mask and have a successor: their tiles run the branch-free
    // body.  The few tiles after that (sequence tail, causal diagonal, idle tail of a causal wave) go
    // through the general path with its run-time case distinctions.
    int h_plain_end = min(nh_w, N / 32);
    if (CAUSAL) h_plain_end = min(h_plain_end, wq0 / 32);
    const int n_plain = h_plain_end > 0 ? (h_plain_end - 1) / 2 : 0;   // tiles j with 2j+2 < h_plain_end

    int j = 0;
    for (; j < n_plain; ++j) {
        sync_and_prefetch(j);
        const int stage_n = (stage + 1) % STAGES;
        const char* s_cur = smem + stage * STAGE_BYTES;
        const char* s_nxt = smem + stage_n * STAGE_BYTES;
        half_step(std::false_type{}, std::true_type{}, Sa, Sb, 2 * j, s_cur + k_lane, s_cur + v_lane);
        half_step(std::false_type{}, std::true_type{}, Sb, Sa, 2 * j + 1, s_nxt + k_lane, s_cur + v_lane);
        stage = stage_n;
    }
    for (; j < nt; ++j) {
        sync_and_prefetch(j);
        const int stage_n = (stage + 1) % STAGES;
        const char* s_cur = smem + stage * STAGE_BYTES;
        const char* s_nxt = smem + stage_n * STAGE_BYTES;
        run_half(Sa, Sb, 2 * j, s_cur + k_lane, s_cur + v_lane);          // T of this tile's second half, U of its first
        run_half(Sb, Sa, 2 * j + 1, s_nxt + k_lane, s_cur + v_lane);      // T of the next tile's first half, U of this tile's second
        stage = stage_n;
    }

    // ---- epilogue: normalise, write O (16-bit) and LSE (natural log)
    uint16_t* oh = o + head_off;
    float* lh = lse + (size_t)bh * N;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const float l_tot = xor32_sum(l_run[mb]);
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

template <int DTYPE, int D, int NW, int MB, int BN, int STAGES, bool CAUSAL>
int launch(const AttnLaunchArgs& a)
{
    constexpr int BM = NW * MB * 32;
    constexpr int smem = STAGES * 2 * BN * D * 2;
    auto kern = attn_fwd_kernel<DTYPE, D, NW, MB, BN, STAGES, CAUSAL>;
    static bool attr_set = false;   // idempotent; a race only repeats the call
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, smem) != hipSuccess)
            return -1;
        attr_set = true;
    }
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
    // the launch's own status, not hipGetLastError(): that one also reports stale errors of unrelated calls
    const hipError_t e = hipLaunchKernel(reinterpret_cast<const void*>(kern), dim3((unsigned)total), dim3(NW * 64),
                                         args, smem, (hipStream_t)a.stream);
    return e == hipSuccess ? 0 : -1;
}

template <int DTYPE, int D>
int launch_d(const AttnLaunchArgs& a)
{
    constexpr int NW = ATTN_CFG_NW, MB = ATTN_CFG_MB, BN = ATTN_CFG_BN, STAGES = ATTN_CFG_STAGES;
    return a.causal ? launch<DTYPE, D, NW, MB, BN, STAGES, true>(a) : launch<DTYPE, D, NW, MB, BN, STAGES, false>(a);
}

}  // namespace

int attn_launch(const AttnLaunchArgs& a)
{
    if (a.dtype == 0) return a.d == 128 ? launch_d<0, 128>(a) : launch_d<0, 64>(a);
    return a.d == 128 ? launch_d<1, 128>(a) : launch_d<1, 64>(a);
}

int attn_launch_tile_param(int d, int causal, int which)
{
    (void)causal;
    if (d != 64 && d != 128) return -1;
    switch (which) {
        case 0: return ATTN_CFG_NW * ATTN_CFG_MB * 32;
        case 1: return ATTN_CFG_BN;
        case 2: return ATTN_CFG_STAGES;
        case 3: return ATTN_CFG_NW * 64;
        default: return -1;
    }
}
