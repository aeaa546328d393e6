/*
 * attn_fwd.h -- C ABI of the gfx950 (MI355X) fused attention forward library.
 *
 * The operation (the paper's Section 3.4.2 names its three stages per key/value
 * tile: T = Q K^T on the matrix cores, C = softmax on the vector ALU, U = P V on
 * the matrix cores; Section 5.4 names the workload, causal and non-causal
 * multi-head attention):
 *
 *     for every batch b and head h, with q_i, k_j, v_j the rows of Q, K, V:
 *       s_ij  = scale * <q_i, k_j>            (causal: key j is visible to query i iff j <= i)
 *       O_i   = sum_j softmax_j(s_ij) * v_j
 *       LSE_i = ln sum_j exp(s_ij)            (natural log of the scaled, masked scores)
 *
 * computed by a single kernel with a streaming (online) softmax: the N x N
 * score matrix is never written to memory.
 *
 * Arguments (identical for every entry point):
 *   q, k, v  DEVICE pointers, read only.  Layout [B][H][N][d], contiguous, d
 *            fastest, 16-bit elements (IEEE binary16 or bfloat16).
 *   o        DEVICE pointer, written.  Same layout and element type as q.  Every
 *            element is overwritten.  Must not overlap q, k or v.
 *   lse      DEVICE pointer, written.  Layout [B][H][N], float32.
 *   B, H     batch size and number of heads, >= 1.
 *   N        sequence length (queries = keys), >= 1; any value, no multiple required.
 *   d        head dimension, 64 or 128.
 *   scale    multiplies the raw dot products; finite and > 0.
 *   causal   0: every key visible; non-zero: key j visible to query i iff j <= i.
 *   stream   a hipStream_t passed as void* (NULL = the default stream).
 *
 * All five pointers must be 16-byte aligned.  The caller owns every buffer; the
 * library allocates nothing, retains nothing and never synchronises: a call
 * validates its arguments on the host, enqueues one kernel on `stream` on the
 * current device and returns.  Calls are thread safe.
 *
 * Return value: ATTN_FWD_OK or a negative error code; attn_fwd_strerror gives
 * its text.  Argument validation happens before any HIP call, so the argument
 * errors can be provoked on a machine without a GPU.  Nothing is enqueued when
 * an error is returned.
 */
#ifndef ATTN_FWD_H
#define ATTN_FWD_H

#ifdef __cplusplus
extern "C" {
#endif

enum {
    ATTN_FWD_OK = 0,
    ATTN_FWD_ERR_NULL = -1,       /* a pointer argument is NULL */
    ATTN_FWD_ERR_SHAPE = -2,      /* B, H or N < 1, or d not in {64, 128}, or unknown dtype */
    ATTN_FWD_ERR_SCALE = -3,      /* scale is NaN, infinite, zero or negative */
    ATTN_FWD_ERR_ALIGN = -4,      /* a pointer is not 16-byte aligned */
    ATTN_FWD_ERR_OVERFLOW = -5,   /* B*H*N*d does not fit the kernel's 32-bit element indexing */
    ATTN_FWD_ERR_LAUNCH = -6,     /* the HIP runtime refused the launch */
    ATTN_FWD_ERR_ALIAS = -7       /* o or lse overlaps q, k, v or each other */
};

enum { ATTN_FWD_FP16 = 0, ATTN_FWD_BF16 = 1 };

/* Q, K, V, O in IEEE binary16. */
int attn_fwd_f16(const void *q, const void *k, const void *v, void *o, float *lse,
                 int B, int H, int N, int d, float scale, int causal, void *stream);

/* Q, K, V, O in bfloat16. */
int attn_fwd_bf16(const void *q, const void *k, const void *v, void *o, float *lse,
                  int B, int H, int N, int d, float scale, int causal, void *stream);

/* Same call with the element type as an argument (ATTN_FWD_FP16 / ATTN_FWD_BF16). */
int attn_fwd(const void *q, const void *k, const void *v, void *o, float *lse,
             int B, int H, int N, int d, float scale, int causal, void *stream, int dtype);

/*
 * The same operation on 8-bit-float inputs, the second precision ("FP8") in which the paper
 * evaluates attention (Section 5.4).  The paper fixes neither the format nor the scaling convention;
 * the reading taken here:
 *   q, k, v  DEVICE pointers, read only, [B][H][N][d] contiguous, ONE byte per element in OCP E4M3
 *            (1 sign, 4 exponent bits with bias 7, 3 fraction bits, largest finite 448, no
 *            infinities, S.1111.111 = NaN): the 8-bit float the gfx950 matrix cores take.  There are
 *            no separate scale tensors: a per-tensor dequantisation factor of Q and of K is folded
 *            into `scale` by the caller, one of V multiplies O afterwards.
 *   o        DEVICE pointer, written, [B][H][N][d] in the 16-bit type out_dtype (ATTN_FWD_FP16 or
 *            ATTN_FWD_BF16); must not overlap q, k or v.
 *   lse      DEVICE pointer, written, [B][H][N] float32.
 * Both contractions run on the 8-bit matrix-core path: the probabilities are rounded to E4M3 (round
 * to nearest even) before P V, accumulation is fp32, and O is normalised by the sum of the ROUNDED
 * probabilities, so every output row is a convex combination of V rows; LSE is the natural log of
 * that same sum (plus the reference maximum).  All other arguments, the alignment rule, ownership,
 * asynchrony and the return codes are those of attn_fwd.
 *
 * Numeric contract of the rounding of P (what a caller, or a test, may rely on).  The probabilities are rounded
 * relative to a per-row reference r that the kernel keeps while it walks the keys: r is a score of the row
 * that has really occurred, never above the running maximum and at most 8 powers of two (a factor 2^8 in the
 * probabilities) below it; it only moves up, by taking the value of the running maximum, when that
 * maximum has grown by more than 2^8 since r was set.  Every weight exp(s - r) <= 2^8 is rounded to E4M3 with
 * round-to-nearest-even: relative error at most 2^-4 for values down to 2^-6 (the smallest normal number),
 * absolute error at most 2^-10 below that (the spacing of the subnormals is 2^-9), zero below 2^-10.  In
 * terms of the exact normalised probabilities p_j of a row the weight given to key j is therefore off by at
 * most min(p_j, max(2^-4 p_j, 2^-10 max_j p_j)) before normalisation; the 2^-10 term is the one that
 * depends on the 2^8 window.
 */
int attn_fwd_fp8(const void *q, const void *k, const void *v, void *o, float *lse,
                 int B, int H, int N, int d, float scale, int causal, void *stream, int out_dtype);

/* Host-only argument check of attn_fwd_fp8. */
int attn_fwd_fp8_check_args(const void *q, const void *k, const void *v, const void *o, const float *lse,
                            int B, int H, int N, int d, float scale, int out_dtype);

/* Launch parameters of the 8-bit-float kernel for head dimension d; `which` as in attn_fwd_tile_param. */
int attn_fwd_fp8_tile_param(int d, int which);

/* Host-only argument check: what the 16-bit entry points above would return before launching. */
int attn_fwd_check_args(const void *q, const void *k, const void *v, const void *o, const float *lse,
                        int B, int H, int N, int d, float scale, int dtype);

/* Static, NUL-terminated description of a return code.  Never NULL. */
const char *attn_fwd_strerror(int code);

/* Library version, major*10000 + minor*100 + patch. */
int attn_fwd_version(void);

/*
 * Name of a launch parameter of the kernel chosen for (d, causal) and its value,
 * for benchmark reports: which = 0 query rows per workgroup (BM), 1 keys per
 * step (BN), 2 LDS stages, 3 threads per workgroup.  Returns -1 for an unknown
 * `which` or unsupported d.
 */
int attn_fwd_tile_param(int d, int causal, int which);

/*
 * The static tile schedule of the launch (host-side copy of what the kernel evaluates; the paper's
 * Section 4.2 describes persistent kernels that walk a tile queue).  A launch covers `total` logical
 * tiles (logical tile t = (batch*head t / nqt, query tile t % nqt), nqt = ceil(N / BM); under the
 * causal mask the query tiles of a head are numbered from the longest to the shortest) with `grid`
 * workgroups, 1 <= grid <= total.  Returns the logical tile workgroup `block` processes in round
 * `round` (0, 1, ...), -1 when it has none in that round or any later one, -2 for arguments out of
 * range.  Every logical tile belongs to exactly one (block, round).
 */
int attn_fwd_tile_schedule(int total, int grid, int block, int round);

/*
 * Measurement aid for the MFMA roofline (not part of the attention path).  Enqueues on `stream` one
 * kernel of `workgroups` workgroups (two waves per SIMD of a CU, like the attention kernel) in which
 * every wave issues iters*8 back-to-back 32x32x16 MFMAs of the given element type on operands held in
 * registers: no memory traffic, no vector work.  random_operands = 0 uses all-zero operands (nothing
 * toggles; the clock stays at its maximum), non-zero uses pseudo-random finite values (the toggling
 * of real inputs; the clock settles where the power management puts it).  The caller times the launch
 * (events on `stream`) and divides attn_fwd_mfma_probe_flops(workgroups, iters) by the duration.
 *   sink   DEVICE pointer, written: attn_fwd_mfma_probe_sink_floats(workgroups) floats, 4-byte aligned.
 * Returns ATTN_FWD_OK, ATTN_FWD_ERR_NULL, ATTN_FWD_ERR_SHAPE (workgroups outside 1..65536, iters outside
 * 1..2^24, unknown dtype), ATTN_FWD_ERR_ALIGN or ATTN_FWD_ERR_LAUNCH; validation precedes any HIP call.
 *
 * dtype may also be ATTN_FWD_PROBE_E4M3: then the stream consists of 32x32x64 MFMAs on 8-bit-float
 * (E4M3) operands, four times the work per instruction (the roofline of attn_fwd_fp8 and gemm_nt_fp8).
 */
enum { ATTN_FWD_PROBE_E4M3 = 2 };
int attn_fwd_mfma_probe(float *sink, int workgroups, int iters, int random_operands, int dtype, void *stream);

/* Floating-point operations one such launch executes with 16-bit operands (0.0 for non-positive arguments). */
double attn_fwd_mfma_probe_flops(int workgroups, int iters);

/* The same for any element type of the probe (0.0 for an unknown dtype). */
double attn_fwd_mfma_probe_flops_of(int workgroups, int iters, int dtype);

/* Number of floats the launch writes to `sink` (-1 for workgroups outside 1..65536). */
int attn_fwd_mfma_probe_sink_floats(int workgroups);

#ifdef __cplusplus
}
#endif

#endif /* ATTN_FWD_H */
