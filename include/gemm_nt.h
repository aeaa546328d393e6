/*
 * gemm_nt.h -- C ABI of the gfx950 (MI355X) matrix product C = A * B^T.
 *
 * The operation is the matrix multiplication the paper uses as its running example and first
 * benchmark (the program of Section 3.1 accumulates the dot product of an [M, K] tile source with the
 * transpose of an [N, K] one; Section 5.2 measures M = N = 8192 with K from 256 to 16384):
 *
 *     C[m][n] = sum_{k=0}^{K-1} A[m][k] * B[n][k]        (fp32 accumulation, result rounded to nearest even)
 *
 * Arguments:
 *   a       DEVICE pointer, read only.  [M][K] row-major (k fastest), 16-bit elements.
 *   b       DEVICE pointer, read only.  [N][K] row-major (k fastest), same element type.
 *   c       DEVICE pointer, written.    [M][N] row-major (n fastest), same element type.  Every element
 *           is overwritten.  Must not overlap a or b.
 *   M, N    >= 1, any value (tiles that overhang the matrix are handled inside the kernel).
 *   K       >= 32 and a multiple of 32 (the K tile of the kernel; the paper's sweep uses 256 ... 16384).
 *   stream  a hipStream_t passed as void* (NULL = the default stream).
 *   dtype   GEMM_NT_FP16 (IEEE binary16) or GEMM_NT_BF16 (bfloat16).
 *
 * a and b must be 16-byte aligned, c 2-byte aligned (8-byte alignment and N % 4 == 0 give the fast
 * stores).  The caller owns every buffer; the library allocates nothing, retains nothing and never
 * synchronises: a call validates its arguments on the host, enqueues one kernel on `stream` on the
 * current device and returns.  Calls are thread safe.
 *
 * Return value: GEMM_NT_OK or a negative error code (gemm_nt_strerror gives its text).  Validation
 * happens before any HIP call; nothing is enqueued when an error is returned.
 */
#ifndef GEMM_NT_H
#define GEMM_NT_H

#ifdef __cplusplus
extern "C" {
#endif

enum {
    GEMM_NT_OK = 0,
    GEMM_NT_ERR_NULL = -1,       /* a pointer argument is NULL */
    GEMM_NT_ERR_SHAPE = -2,      /* M or N < 1, K < 32 or not a multiple of 32, or unknown dtype */
    GEMM_NT_ERR_ALIGN = -4,      /* a or b not 16-byte aligned, or c not 2-byte aligned */
    GEMM_NT_ERR_OVERFLOW = -5,   /* M*K, N*K or M*N elements do not fit the kernel's 32-bit byte offsets */
    GEMM_NT_ERR_LAUNCH = -6,     /* the HIP runtime refused the launch */
    GEMM_NT_ERR_ALIAS = -7       /* c overlaps a or b */
};

enum { GEMM_NT_FP16 = 0, GEMM_NT_BF16 = 1 };

int gemm_nt(const void *a, const void *b, void *c, int M, int N, int K, void *stream, int dtype);

/*
 * The same call with the kernel configuration chosen by the caller instead of by K (for tests and
 * measurements; every configuration computes the same product): 0 = as gemm_nt, 1 = 8 waves of 128 x 64,
 * 2 = the same with the copies of two consecutive K tiles issued together, 3 = 4 waves of 128 x 128,
 * 4 = the same with paired copies.  GEMM_NT_ERR_SHAPE for any other value.
 */
int gemm_nt_config(const void *a, const void *b, void *c, int M, int N, int K, void *stream, int dtype, int config);

/* The same call with the element type in the name. */
int gemm_nt_f16(const void *a, const void *b, void *c, int M, int N, int K, void *stream);
int gemm_nt_bf16(const void *a, const void *b, void *c, int M, int N, int K, void *stream);

/* Host-only argument check: what gemm_nt would return before launching. */
int gemm_nt_check_args(const void *a, const void *b, const void *c, int M, int N, int K, int dtype);

/*
 * The product of 8-bit-float operands: the paper measures its matrix multiplication in FP16 and in FP8
 * (Section 5.2, M = N = 8192, K from 256 to 16384).
 *
 *   a, b       DEVICE pointers, read only, [M][K] and [N][K] row-major bytes in the OCP E4M3 format
 *              (1 sign, 4 exponent bits with bias 7, 3 fraction bits; no infinities, S.1111.111 is NaN).
 *   c          DEVICE pointer, written, [M][N] row-major 16-bit elements of type out_dtype.  Every element
 *              is overwritten.  Must not overlap a or b.
 *   K          >= 64 and a multiple of 64 (the K tile of this kernel).
 *   out_dtype  GEMM_NT_FP16 or GEMM_NT_BF16.
 *
 * The products of two E4M3 values are exact; they are summed in fp32 on the matrix cores (64 products per
 * instruction, added to the running fp32 sum) and the result is rounded to nearest even once.  Alignment,
 * ownership, stream semantics, thread safety and error codes are those of gemm_nt; GEMM_NT_ERR_SHAPE also
 * covers K < 64 or K not a multiple of 64, GEMM_NT_ERR_OVERFLOW M*K or N*K >= 2^31 bytes.
 */
int gemm_nt_fp8(const void *a, const void *b, void *c, int M, int N, int K, void *stream, int out_dtype);

/*
 * The same call with the kernel configuration chosen by the caller instead of by K (for tests and
 * measurements; every configuration computes the same product): 0 = as gemm_nt_fp8, 1 = 8 waves of 128 x 64,
 * 2 = the same with the copies of two consecutive K tiles issued together, 3 = 4 waves of 128 x 128,
 * 4 = the same with paired copies.  GEMM_NT_ERR_SHAPE for any other value.
 */
int gemm_nt_fp8_config(const void *a, const void *b, void *c, int M, int N, int K, void *stream, int out_dtype, int config);

/* Host-only argument check: what gemm_nt_fp8 would return before launching. */
int gemm_nt_fp8_check_args(const void *a, const void *b, const void *c, int M, int N, int K, int out_dtype);

/* Static, NUL-terminated description of a return code.  Never NULL. */
const char *gemm_nt_strerror(int code);

/*
 * Launch parameters of the kernel, for benchmark reports: which = 0 rows of C per workgroup, 1 columns,
 * 2 K tile, 3 LDS stages, 4 threads per workgroup.  Returns -1 for an unknown `which`.
 */
int gemm_nt_tile_param(int which);

/* The same for the kernel behind gemm_nt_fp8 (the configuration a large K takes). */
int gemm_nt_fp8_tile_param(int which);

#ifdef __cplusplus
}
#endif

#endif /* GEMM_NT_H */
