// Host side of the C ABI declared in include/gemm_nt.h: argument validation (before any HIP call, so
// the error paths run on a machine without a GPU) and dispatch to the kernel launcher.
#include "gemm_nt.h"

#include <cstdint>

#include "gemm_launch.h"

namespace {

bool overlaps(const void* a, unsigned long long na, const void* b, unsigned long long nb)
{
    const auto pa = reinterpret_cast<std::uintptr_t>(a), pb = reinterpret_cast<std::uintptr_t>(b);
    return pa < pb + nb && pb < pa + na;
}

}  // namespace

extern "C" {

int gemm_nt_check_args(const void* a, const void* b, const void* c, int M, int N, int K, int dtype)
{
    if (!a || !b || !c) return GEMM_NT_ERR_NULL;
    if (M < 1 || N < 1 || K < 32 || K % 32 != 0) return GEMM_NT_ERR_SHAPE;
    if (dtype != GEMM_NT_FP16 && dtype != GEMM_NT_BF16) return GEMM_NT_ERR_SHAPE;
    if ((reinterpret_cast<std::uintptr_t>(a) | reinterpret_cast<std::uintptr_t>(b)) & 15u) return GEMM_NT_ERR_ALIGN;
    if (reinterpret_cast<std::uintptr_t>(c) & 1u) return GEMM_NT_ERR_ALIGN;
    // per-lane byte offsets inside an operand are 32-bit; tile counts are ints
    const unsigned long long a_bytes = 2ull * (unsigned long long)M * (unsigned long long)K;
    const unsigned long long b_bytes = 2ull * (unsigned long long)N * (unsigned long long)K;
    const unsigned long long c_bytes = 2ull * (unsigned long long)M * (unsigned long long)N;
    if (a_bytes >= (1ull << 31) || b_bytes >= (1ull << 31) || c_bytes >= (1ull << 33)) return GEMM_NT_ERR_OVERFLOW;
    if (overlaps(c, c_bytes, a, a_bytes) || overlaps(c, c_bytes, b, b_bytes)) return GEMM_NT_ERR_ALIAS;
    return GEMM_NT_OK;
}

int gemm_nt_config(const void* a, const void* b, void* c, int M, int N, int K, void* stream, int dtype, int config)
{
    const int rc = gemm_nt_check_args(a, b, c, M, N, K, dtype);
    if (rc != GEMM_NT_OK) return rc;
    if (config < 0 || config > 4) return GEMM_NT_ERR_SHAPE;
    GemmLaunchArgs g{a, b, c, M, N, K, dtype, stream, config};
    return gemm_launch(g) == 0 ? GEMM_NT_OK : GEMM_NT_ERR_LAUNCH;
}

int gemm_nt(const void* a, const void* b, void* c, int M, int N, int K, void* stream, int dtype)
{
    return gemm_nt_config(a, b, c, M, N, K, stream, dtype, 0);
}

int gemm_nt_fp8_check_args(const void* a, const void* b, const void* c, int M, int N, int K, int out_dtype)
{
    if (!a || !b || !c) return GEMM_NT_ERR_NULL;
    if (M < 1 || N < 1 || K < 64 || K % 64 != 0) return GEMM_NT_ERR_SHAPE;
    if (out_dtype != GEMM_NT_FP16 && out_dtype != GEMM_NT_BF16) return GEMM_NT_ERR_SHAPE;
    if ((reinterpret_cast<std::uintptr_t>(a) | reinterpret_cast<std::uintptr_t>(b)) & 15u) return GEMM_NT_ERR_ALIGN;
    if (reinterpret_cast<std::uintptr_t>(c) & 1u) return GEMM_NT_ERR_ALIGN;
    const unsigned long long a_bytes = (unsigned long long)M * (unsigned long long)K;
    const unsigned long long b_bytes = (unsigned long long)N * (unsigned long long)K;
    const unsigned long long c_bytes = 2ull * (unsigned long long)M * (unsigned long long)N;
    if (a_bytes >= (1ull << 31) || b_bytes >= (1ull << 31) || c_bytes >= (1ull << 33)) return GEMM_NT_ERR_OVERFLOW;
    if (overlaps(c, c_bytes, a, a_bytes) || overlaps(c, c_bytes, b, b_bytes)) return GEMM_NT_ERR_ALIAS;
    return GEMM_NT_OK;
}

int gemm_nt_fp8_config(const void* a, const void* b, void* c, int M, int N, int K, void* stream, int out_dtype, int config)
{
    const int rc = gemm_nt_fp8_check_args(a, b, c, M, N, K, out_dtype);
    if (rc != GEMM_NT_OK) return rc;
    if (config < 0 || config > 4) return GEMM_NT_ERR_SHAPE;
    GemmLaunchArgs g{a, b, c, M, N, K, out_dtype, stream, config};
    return gemm_fp8_launch(g) == 0 ? GEMM_NT_OK : GEMM_NT_ERR_LAUNCH;
}

int gemm_nt_fp8(const void* a, const void* b, void* c, int M, int N, int K, void* stream, int out_dtype)
{
    return gemm_nt_fp8_config(a, b, c, M, N, K, stream, out_dtype, 0);
}

int gemm_nt_f16(const void* a, const void* b, void* c, int M, int N, int K, void* stream)
{
    return gemm_nt(a, b, c, M, N, K, stream, GEMM_NT_FP16);
}

int gemm_nt_bf16(const void* a, const void* b, void* c, int M, int N, int K, void* stream)
{
    return gemm_nt(a, b, c, M, N, K, stream, GEMM_NT_BF16);
}

const char* gemm_nt_strerror(int code)
{
    switch (code) {
        case GEMM_NT_OK: return "success";
        case GEMM_NT_ERR_NULL: return "a pointer argument is NULL";
        case GEMM_NT_ERR_SHAPE: return "unsupported shape or dtype (need M,N >= 1, K a multiple of 32 -- 64 for 8-bit operands --, dtype in {0,1})";
        case GEMM_NT_ERR_ALIGN: return "a and b must be 16-byte aligned, c 2-byte aligned";
        case GEMM_NT_ERR_OVERFLOW: return "matrix too large for the kernel's index arithmetic";
        case GEMM_NT_ERR_LAUNCH: return "HIP refused the kernel launch";
        case GEMM_NT_ERR_ALIAS: return "c overlaps a or b";
        default: return "unknown error code";
    }
}

int gemm_nt_tile_param(int which) { return gemm_launch_tile_param(which); }

int gemm_nt_fp8_tile_param(int which) { return gemm_fp8_launch_tile_param(which); }

}  // extern "C"
