/*
 * attn_ref.c -- CPU oracle for scaled-dot-product attention forward.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It is never called from the product path;
 * it shares no code, header, table or helper with the HIP kernels.
 *
 * What it computes (the paper's Section 3.4.2 names the three stages of the
 * attention iteration -- T = Q K^T, C = softmax, U = P V -- and Section 5.4
 * names the workload "(non-)causal multi-head attention"; the arithmetic is
 * the textbook definition the paper cites for attention):
 *
 *   for every batch b and head h independently, with q_i, k_j, v_j the rows of
 *   the [N, d] matrices Q, K, V decoded exactly from their 16-bit patterns:
 *
 *     s_ij  = scale * sum_t q_it * k_jt          (causal: s_ij = -inf for j > i)
 *     M_i   = max_j s_ij
 *     Z_i   = sum_j exp(s_ij - M_i)
 *     p_ij  = exp(s_ij - M_i) / Z_i
 *     O_i   = sum_j p_ij * v_j
 *     LSE_i = M_i + ln Z_i                       (natural log)
 *
 * Everything is fp64.  The full-tensor entry point materialises the whole
 * N x N score matrix of a head before it normalises it; the row-sampled entry
 * point does the same for single query rows (a 1 x N score row) so that the
 * full-size workloads can be checked on sampled outputs.
 *
 * No blocking, fusion, streaming softmax or reordering: a reader can check it
 * against the definition by eye.  Threads (OpenMP) split the query rows only.
 *
 * Layout: q, k, v are [B][H][N][d], d fastest, raw storage patterns: uint16
 * for fp16 and bf16, uint8 for the 8-bit float (OCP E4M3, the "fp8" of the
 * paper's second attention precision, Section 5.4); o is [B][H][N][d] double;
 * lse is [B][H][N] double.  The element type only selects the decoder: the
 * arithmetic above is the same for all three.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define ATTN_REF_FP16 0
#define ATTN_REF_BF16 1
#define ATTN_REF_E4M3 2

/* IEEE-754 binary16 -> double, exact.  1 sign, 5 exponent (bias 15), 10 fraction bits. */
static double decode_fp16(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int f = h & 0x3ff;
    double mag;
    if (e == 0)
        mag = ldexp((double)f, -24);               /* zero and subnormals: f * 2^-10 * 2^-14 */
    else if (e == 31)
        mag = f ? NAN : INFINITY;
    else
        mag = ldexp(1.0 + (double)f / 1024.0, e - 15);
    return sign ? -mag : mag;
}

/* bfloat16 -> double, exact.  1 sign, 8 exponent (bias 127), 7 fraction bits. */
static double decode_bf16(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 7) & 0xff;
    int f = h & 0x7f;
    double mag;
    if (e == 0)
        mag = ldexp((double)f, -133);              /* f * 2^-7 * 2^-126 */
    else if (e == 255)
        mag = f ? NAN : INFINITY;
    else
        mag = ldexp(1.0 + (double)f / 128.0, e - 127);
    return sign ? -mag : mag;
}

/*
 * OCP 8-bit float E4M3 ("e4m3fn") -> double, exact.  1 sign, 4 exponent (bias 7), 3 fraction bits;
 * no infinities: exponent 15 is an ordinary binade (up to 1.75 * 2^8 = 448) except that the
 * all-ones pattern S.1111.111 is NaN.
 */
static double decode_e4m3(uint8_t b)
{
    int sign = (b >> 7) & 1;
    int e = (b >> 3) & 0xf;
    int f = b & 0x7;
    double mag;
    if (e == 0)
        mag = ldexp((double)f, -9);                /* zero and subnormals: f * 2^-3 * 2^-6 */
    else if (e == 15 && f == 7)
        mag = NAN;
    else
        mag = ldexp(1.0 + (double)f / 8.0, e - 7);
    return sign ? -mag : mag;
}

static int valid_dtype(int dtype)
{
    return dtype == ATTN_REF_FP16 || dtype == ATTN_REF_BF16 || dtype == ATTN_REF_E4M3;
}

/* Element `idx` of a tensor stored in the given element type. */
static double decode_at(const void *base, long idx, int dtype)
{
    if (dtype == ATTN_REF_E4M3) return decode_e4m3(((const uint8_t *)base)[idx]);
    uint16_t h = ((const uint16_t *)base)[idx];
    return dtype == ATTN_REF_BF16 ? decode_bf16(h) : decode_fp16(h);
}

/* Exported so that the decoders themselves can be pinned over all their patterns. */
void attn_ref_decode(const void *src, double *dst, long n, int dtype)
{
    for (long i = 0; i < n; ++i) dst[i] = decode_at(src, i, dtype);
}

static int resolve_threads(int nthreads)
{
#ifdef _OPENMP
    if (nthreads <= 0) nthreads = omp_get_max_threads();
#else
    nthreads = 1;
#endif
    return nthreads;
}

int attn_ref_max_threads(void)
{
    return resolve_threads(0);
}

/*
 * One query row against all keys of its head, from already-decoded matrices.
 *   qrow: [d]; K, V: [N][d]; srow: scratch [N] that receives the score row;
 *   orow: [d] out; returns LSE of the row.
 */
static double attend_row(const double *qrow, const double *K, const double *V, double *srow,
                         double *orow, long i, long N, long d, double scale, int causal)
{
    /* scores of row i */
    for (long j = 0; j < N; ++j) {
        if (causal && j > i) {
            srow[j] = -INFINITY;
        } else {
            double acc = 0.0;
            for (long t = 0; t < d; ++t) acc += qrow[t] * K[j * d + t];
            srow[j] = scale * acc;
        }
    }
    /* softmax of the row */
    double M = -INFINITY;
    for (long j = 0; j < N; ++j)
        if (srow[j] > M) M = srow[j];
    double Z = 0.0;
    for (long j = 0; j < N; ++j) {
        srow[j] = exp(srow[j] - M);                /* exp(-inf) = 0 for masked keys */
        Z += srow[j];
    }
    for (long j = 0; j < N; ++j) srow[j] /= Z;
    /* weighted sum of the value rows */
    for (long t = 0; t < d; ++t) orow[t] = 0.0;
    for (long j = 0; j < N; ++j) {
        double p = srow[j];
        if (p == 0.0) continue;
        for (long t = 0; t < d; ++t) orow[t] += p * V[j * d + t];
    }
    return M + log(Z);
}

/*
 * Full attention forward in fp64.  Returns 0, or -1 on bad arguments, -2 when
 * the score matrix cannot be allocated.
 * If p_out is not NULL it receives the normalised probabilities
 * [B][H][N][N] (only sensible for small N; used by the row-sum pin).
 */
int attn_ref_f64(const void *q, const void *k, const void *v, int dtype,
                 double *o, double *lse, double *p_out,
                 int B, int H, int N, int d, double scale, int causal, int nthreads)
{
    if (!q || !k || !v || !o || !lse) return -1;
    if (B <= 0 || H <= 0 || N <= 0 || d <= 0) return -1;
    if (!valid_dtype(dtype)) return -1;
    nthreads = resolve_threads(nthreads);

    const long n = N, dd = d;
    double *Q = malloc(sizeof(double) * n * dd);
    double *K = malloc(sizeof(double) * n * dd);
    double *V = malloc(sizeof(double) * n * dd);
    double *S = malloc(sizeof(double) * n * n);    /* the head's full score matrix */
    if (!Q || !K || !V || !S) {
        free(Q); free(K); free(V); free(S);
        return -2;
    }

    for (long bh = 0; bh < (long)B * H; ++bh) {
        const long head = bh * n * dd;             /* first element of this head */
        for (long e = 0; e < n * dd; ++e) {
            Q[e] = decode_at(q, head + e, dtype);
            K[e] = decode_at(k, head + e, dtype);
            V[e] = decode_at(v, head + e, dtype);
        }
        double *oh = o + bh * n * dd;
        double *lh = lse + bh * n;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 8) num_threads(nthreads)
#endif
        for (long i = 0; i < n; ++i) {
            lh[i] = attend_row(Q + i * dd, K, V, S + i * n, oh + i * dd, i, n, dd, scale, causal);
        }
        if (p_out) {
            double *ph = p_out + bh * n * n;
            for (long e = 0; e < n * n; ++e) ph[e] = S[e];
        }
    }
    free(Q); free(K); free(V); free(S);
    return 0;
}

/*
 * The same definition for sampled query rows: rows[r] = {b, h, i} (3 ints per
 * sample); o_rows is [nrows][d], lse_rows is [nrows]; p_rows, when not NULL,
 * receives the rows' normalised probabilities [nrows][N].  Used to check the
 * full-size workloads, where all B*H*N rows would take the CPU minutes.
 */
int attn_ref_rows_f64(const void *q, const void *k, const void *v, int dtype,
                      const int *rows, int nrows, double *o_rows, double *lse_rows, double *p_rows,
                      int B, int H, int N, int d, double scale, int causal, int nthreads)
{
    if (!q || !k || !v || !rows || !o_rows || !lse_rows) return -1;
    if (B <= 0 || H <= 0 || N <= 0 || d <= 0 || nrows < 0) return -1;
    if (!valid_dtype(dtype)) return -1;
    for (int r = 0; r < nrows; ++r) {
        if (rows[3 * r] < 0 || rows[3 * r] >= B || rows[3 * r + 1] < 0 || rows[3 * r + 1] >= H ||
            rows[3 * r + 2] < 0 || rows[3 * r + 2] >= N)
            return -1;
    }
    nthreads = resolve_threads(nthreads);
    const long n = N, dd = d;
    int status = 0;
#ifdef _OPENMP
#pragma omp parallel num_threads(nthreads)
#endif
    {
        double *K = malloc(sizeof(double) * n * dd);
        double *V = malloc(sizeof(double) * n * dd);
        double *Qr = malloc(sizeof(double) * dd);
        double *srow = malloc(sizeof(double) * n);
        if (!K || !V || !Qr || !srow) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
            status = -2;
        } else {
#ifdef _OPENMP
#pragma omp for schedule(dynamic, 1)
#endif
            for (int r = 0; r < nrows; ++r) {
                long b = rows[3 * r], h = rows[3 * r + 1], i = rows[3 * r + 2];
                long bh = b * H + h;
                const long head = bh * n * dd;
                for (long e = 0; e < n * dd; ++e) {
                    K[e] = decode_at(k, head + e, dtype);
                    V[e] = decode_at(v, head + e, dtype);
                }
                for (long t = 0; t < dd; ++t) Qr[t] = decode_at(q, head + i * dd + t, dtype);
                lse_rows[r] = attend_row(Qr, K, V, srow, o_rows + (long)r * dd, i, n, dd, scale, causal);
                if (p_rows)                        /* the row's normalised probabilities */
                    for (long j = 0; j < n; ++j) p_rows[(long)r * n + j] = srow[j];
            }
        }
        free(K); free(V); free(Qr); free(srow);
    }
    return status;
}
