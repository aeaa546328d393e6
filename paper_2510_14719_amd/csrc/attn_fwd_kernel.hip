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

#include "attn_launch.h"

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

#define LDS_AS __attribute__((address_space(3)))

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
    constexpr int KB = BN / 32;                 // 32-key blocks per K/V tile
    constexpr int KK = D / 16;                  // contraction steps of Q K^T
    constexpr int DB = D / 32;                  // 32-wide feature blocks of O
    constexpr int ROW_BYTES = D * 2;
    constexpr int TILE_BYTES = BN * ROW_BYTES;  // one K or one V tile
    constexpr int STAGE_BYTES = 2 * TILE_BYTES;
    constexpr int RB = BN / 16;                 // 16-row blocks per tile
    constexpr int CHUNKS = TILE_BYTES / 1024;   // 1 KiB wave-transfers per tile
    constexpr int CPW = CHUNKS / NW;            // ... per wave
    static_assert(CHUNKS % NW == 0, "tile must split evenly over the waves");
    static_assert(STAGES >= 3, "prefetch distance 2 needs three stages");

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
    const uint16_t* kh = k + head_off;
    const uint16_t* vh = v + head_off;

    // ---- number of K/V tiles
    int nt = (N + BN - 1) / BN;
    if (CAUSAL) {
        const int last_q = min(q0 + BM, N) - 1;
        nt = min(nt, last_q / BN + 1);
    }

    // ---- per-lane constants of the global -> LDS copies
    // K tile in LDS: [feature group of 32][16-row block][16-byte column of the group (4)][row (16)][16 B]
    // V tile in LDS: [feature group of 32][row (BN)][64 B]
    int k_row[CPW], k_col[CPW], v_row[CPW], v_col[CPW];
    unsigned k_dst[CPW], v_dst[CPW];
#pragma unroll
    for (int i = 0; i < CPW; ++i) {
        const int wc = wave * CPW + i;
        const int fg = wc / RB, rb = wc % RB;
        k_row[i] = rb * 16 + (lane & 15);
        k_col[i] = (fg * 4 + (lane >> 4)) * 16;
        v_row[i] = rb * 16 + (lane >> 2);
        v_col[i] = fg * 64 + (lane & 3) * 16;
        k_dst[i] = lds_base + wc * 1024;
        v_dst[i] = lds_base + TILE_BYTES + wc * 1024;
    }
    auto issue_tile = [&](int t, int stage) {
        const int kv0 = t * BN;
        const unsigned sbase = stage * STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < CPW; ++i) {
            const int rk = min(kv0 + k_row[i], N - 1);
            dma16(kh, (unsigned)(rk * ROW_BYTES + k_col[i]), k_dst[i] + sbase);
        }
#pragma unroll
        for (int i = 0; i < CPW; ++i) {
            const int rv = min(kv0 + v_row[i], N - 1);
            dma16(vh, (unsigned)(rv * ROW_BYTES + v_col[i]), v_dst[i] + sbase);
        }
    };

    // ---- prologue: two tiles in flight, Q fragments into registers
    issue_tile(0, 0);
    if (nt > 1) issue_tile(1, 1);

    s16x8 Qf[MB][KK];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const int row = min(wq0 + mb * 32 + lr, N - 1);
        const uint16_t* qr = qh + (size_t)row * D;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk)
            Qf[mb][kk] = *reinterpret_cast<const s16x8*>(qr + (kk * 2 + g) * 8);
    }

    f32x16 O[MB][DB];
    float m_run[MB], l_run[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        m_run[mb] = -__builtin_inff();
        l_run[mb] = 0.f;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) O[mb][db][i] = 0.f;
    }

    // per-lane LDS read offsets (the rest of every address is an immediate)
    const int k_lane = (lr >> 4) * 1024 + g * 256 + (lr & 15) * 16;
    const int v_lane = TILE_BYTES + (4 * g + ((lane & 15) >> 2)) * 64 + ((lane >> 4) & 1) * 32 + (lane & 3) * 8;

    int stage = 0;
    for (int j = 0; j < nt; ++j) {
        // tile j has landed (this wave's share), then everybody's share; the barrier also says that
        // every wave is done reading tile j-1, whose stage the next copy overwrites
        if (j + 1 < nt) wait_vmcnt<2 * CPW>(); else wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();
        if (j + 2 < nt) {
            int s2 = stage + 2; if (s2 >= STAGES) s2 -= STAGES;
            issue_tile(j + 2, s2);
        }
        const int kv0 = j * BN;
        const char* sk = smem + stage * STAGE_BYTES + k_lane;
        const char* sv = smem + stage * STAGE_BYTES + v_lane;
        stage = (stage + 1 == STAGES) ? 0 : stage + 1;

        if (CAUSAL && kv0 > wq0 + MB * 32 - 1) continue;   // every key of the tile is hidden from this wave

        // ---- T: S^T = K Q^T
        f32x16 S[MB][KB];
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {
                const s16x8 kf = *reinterpret_cast<const s16x8*>(sk + ((kk >> 1) * RB + kb * 2) * 1024 + (kk & 1) * 512);
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    if (kk == 0) {
                        f32x16 z;
#pragma unroll
                        for (int i = 0; i < 16; ++i) z[i] = 0.f;
                        S[mb][kb] = E::mfma(kf, Qf[mb][kk], z);
                    } else {
                        S[mb][kb] = E::mfma(kf, Qf[mb][kk], S[mb][kb]);
                    }
                }
            }
        }

        // ---- mask: keys past the end of the sequence, and keys after the query when causal
        const bool need_mask = (kv0 + BN > N) || (CAUSAL && kv0 + BN - 1 > wq0);
        if (need_mask) {
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

        // ---- C: streaming softmax (base-2 exponentials, scale folded into the exponent)
        s16x8 Pf[MB][KB][2];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            float mx = S[mb][0][0];
#pragma unroll
            for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                for (int i = 0; i < 16; ++i) mx = __builtin_fmaxf(mx, S[mb][kb][i]);
            mx = xor32_max(mx);
            const float m_new = __builtin_fmaxf(m_run[mb], mx);
            const float alpha = __builtin_amdgcn_exp2f((m_run[mb] - m_new) * scale_log2e);
            const float neg_mc = -m_new * scale_log2e;
            m_run[mb] = m_new;
            float sum = 0.f;
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) {
                float p[16];
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    p[i] = __builtin_amdgcn_exp2f(__builtin_fmaf(S[mb][kb][i], scale_log2e, neg_mc));
                    sum += p[i];
                }
#pragma unroll
                for (int ks = 0; ks < 2; ++ks) {
                    u32x4 w;
#pragma unroll
                    for (int t = 0; t < 4; ++t) w[t] = E::pack2(p[ks * 8 + 2 * t], p[ks * 8 + 2 * t + 1]);
                    Pf[mb][kb][ks] = __builtin_bit_cast(s16x8, w);
                }
            }
            l_run[mb] = l_run[mb] * alpha + sum;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int i = 0; i < 16; ++i) O[mb][db][i] *= alpha;
        }

        // ---- U: O^T += V^T P^T
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    const char* a = sv + db * (BN * 64) + (kb * 32 + ks * 16) * 64;
                    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(a));
                    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(a + 8 * 64));
                    const s16x8 vf = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb) O[mb][db] = E::mfma(vf, Pf[mb][kb][ks], O[mb][db]);
                }
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
