/*
 * gemm_ref.c -- CPU oracle of the "NT" matrix product  C = A * B^T.
 *
 * TEST INFRASTRUCTURE ONLY.  Used by tests/, the smoke test and the cpu_baseline leg of the benchmark;
 * the GPU library neither links nor calls it, and it shares no code with the GPU path (it has its own
 * decoders).
 *
 * What it computes is the plain definition of the product the paper's matrix-multiplication program
 * states (the Triton GEMM of Section 3.1 accumulates dot(a, b^T) over K tiles, with a an [M, K] tile
 * source and b an [N, K] one; Section 5.2 names the workload, M = N = 8192 with K from 256 to 16384):
 *
 *     C[m][n] = sum_{k=0}^{K-1} A[m][k] * B[n][k]
 *
 * with A [M][K] and B [N][K] row-major inputs decoded exactly, every product and the sum in fp64, in
 * the order k = 0, 1, ..., K-1.  The result stays in fp64 (not rounded).  Element types: fp16 (0) and
 * bf16 (1), stored as uint16; the 8-bit float OCP E4M3 (2), stored as uint8 -- the paper evaluates the
 * matrix product in FP16 and in FP8 (Section 5.2).  The type only selects the decoder.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double dec_f16(uint16_t h)
{
    const int sign = h >> 15, e = (h >> 10) & 0x1f, f = h & 0x3ff;
    double v;
    if (e == 0) v = ldexp((double)f, -24);                 /* zero and subnormals */
    else if (e == 31) v = f ? NAN : INFINITY;
    else v = ldexp((double)(f | 0x400), e - 25);
    return sign ? -v : v;
}

static double dec_bf16(uint16_t h)
{
    const uint32_t u = (uint32_t)h << 16;                  /* bfloat16 is the upper half of a binary32 */
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* OCP E4M3: 1 sign, 4 exponent bits (bias 7), 3 fraction bits; no infinities, S.1111.111 is NaN. */
static double dec_e4m3(uint8_t b)
{
    const int sign = b >> 7, e = (b >> 3) & 0xf, f = b & 0x7;
    double v;
    if (e == 0) v = ldexp((double)f, -9);                  /* zero and subnormals */
    else if (e == 15 && f == 7) v = NAN;
    else v = ldexp((double)(f | 0x8), e - 10);
    return sign ? -v : v;
}

/* Element i of a matrix stored in the given type. */
static double dec(const void *base, long i, int dtype)
{
    if (dtype == 2) return dec_e4m3(((const uint8_t *)base)[i]);
    const uint16_t h = ((const uint16_t *)base)[i];
    return dtype == 1 ? dec_bf16(h) : dec_f16(h);
}

static int valid_dtype(int dtype) { return dtype == 0 || dtype == 1 || dtype == 2; }

void gemm_ref_decode(const void *bits, double *out, long n, int dtype)
{
    for (long i = 0; i < n; ++i) out[i] = dec(bits, i, dtype);
}

int gemm_ref_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Full product.  a: [M][K], b: [N][K], c: [M][N] (fp64).  Returns 0, or -1 for bad arguments. */
int gemm_ref_nt_f64(const void *a, const void *b, int dtype, double *c, int M, int N, int K, int nthreads)
{
    if (!a || !b || !c || M < 1 || N < 1 || K < 1 || !valid_dtype(dtype)) return -1;
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#else
    (void)nthreads;
#endif
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m) {
        for (int n = 0; n < N; ++n) {
            double s = 0.0;
            for (int k = 0; k < K; ++k) s += dec(a, (long)m * K + k, dtype) * dec(b, (long)n * K + k, dtype);
            c[(long)m * N + n] = s;
        }
    }
    return 0;
}

/* The same definition for `count` sampled entries idx = {m_0, n_0, m_1, n_1, ...}; out[i] = C[m_i][n_i]. */
int gemm_ref_nt_samples_f64(const void *a, const void *b, int dtype, const int *idx, int count, double *out,
                            int M, int N, int K)
{
    if (!a || !b || !idx || !out || M < 1 || N < 1 || K < 1 || count < 0 || !valid_dtype(dtype)) return -1;
    for (int i = 0; i < count; ++i)
        if (idx[2 * i] < 0 || idx[2 * i] >= M || idx[2 * i + 1] < 0 || idx[2 * i + 1] >= N) return -1;
#pragma omp parallel for schedule(static)
    for (int i = 0; i < count; ++i) {
        const long m = idx[2 * i], n = idx[2 * i + 1];
        double s = 0.0;
        for (int k = 0; k < K; ++k) s += dec(a, m * K + k, dtype) * dec(b, n * K + k, dtype);
        out[i] = s;
    }
    return 0;
}
