// Host side of the C ABI declared in include/attn_fwd.h: argument validation (no HIP call is made
// before the arguments are known to be good, so the error paths run on a machine without a GPU)
// and dispatch to the kernel launcher.
#include "attn_fwd.h"

#include <cmath>
#include <cstdint>

#include "attn_launch.h"
#include "tile_schedule.h"

namespace {

bool overlaps(const void* a, unsigned long long na, const void* b, unsigned long long nb)
{
    const auto pa = reinterpret_cast<std::uintptr_t>(a), pb = reinterpret_cast<std::uintptr_t>(b);
    return pa < pb + nb && pb < pa + na;
}

}  // namespace

extern "C" {

int attn_fwd_check_args(const void* q, const void* k, const void* v, const void* o, const float* lse,
                        int B, int H, int N, int d, float scale, int dtype)
{
    if (!q || !k || !v || !o || !lse) return ATTN_FWD_ERR_NULL;
    if (B < 1 || H < 1 || N < 1 || (d != 64 && d != 128)) return ATTN_FWD_ERR_SHAPE;
    if (dtype != ATTN_FWD_FP16 && dtype != ATTN_FWD_BF16) return ATTN_FWD_ERR_SHAPE;
    if (!std::isfinite(scale) || !(scale > 0.0f)) return ATTN_FWD_ERR_SCALE;
    const std::uintptr_t mis = reinterpret_cast<std::uintptr_t>(q) | reinterpret_cast<std::uintptr_t>(k) |
                               reinterpret_cast<std::uintptr_t>(v) | reinterpret_cast<std::uintptr_t>(o) |
                               reinterpret_cast<std::uintptr_t>(lse);
    if (mis & 15u) return ATTN_FWD_ERR_ALIGN;
    // The kernel indexes inside one head with 32-bit byte offsets and numbers its workgroups with an int.
    const unsigned long long head_bytes = 2ull * (unsigned long long)N * (unsigned long long)d;
    if (head_bytes >= (1ull << 31)) return ATTN_FWD_ERR_OVERFLOW;
    const int bm = attn_launch_tile_param(d, 0, 0);
    const unsigned long long tiles = ((unsigned long long)N + bm - 1) / bm * (unsigned long long)B * (unsigned long long)H;
    if (tiles >= (1ull << 31)) return ATTN_FWD_ERR_OVERFLOW;
    const unsigned long long bytes = head_bytes * (unsigned long long)B * (unsigned long long)H;
    const unsigned long long lse_bytes = 4ull * (unsigned long long)N * (unsigned long long)B * (unsigned long long)H;
    if (overlaps(o, bytes, q, bytes) || overlaps(o, bytes, k, bytes) || overlaps(o, bytes, v, bytes)) return ATTN_FWD_ERR_ALIAS;
    if (overlaps(lse, lse_bytes, q, bytes) || overlaps(lse, lse_bytes, k, bytes) || overlaps(lse, lse_bytes, v, bytes) ||
        overlaps(lse, lse_bytes, o, bytes)) return ATTN_FWD_ERR_ALIAS;
    return ATTN_FWD_OK;
}

int attn_fwd(const void* q, const void* k, const void* v, void* o, float* lse,
             int B, int H, int N, int d, float scale, int causal, void* stream, int dtype)
{
    const int rc = attn_fwd_check_args(q, k, v, o, lse, B, H, N, d, scale, dtype);
    if (rc != ATTN_FWD_OK) return rc;
    AttnLaunchArgs a{q, k, v, o, lse, B, H, N, d, scale, causal != 0, dtype, stream};
    return attn_launch(a) == 0 ? ATTN_FWD_OK : ATTN_FWD_ERR_LAUNCH;
}

int attn_fwd_f16(const void* q, const void* k, const void* v, void* o, float* lse,
                 int B, int H, int N, int d, float scale, int causal, void* stream)
{
    return attn_fwd(q, k, v, o, lse, B, H, N, d, scale, causal, stream, ATTN_FWD_FP16);
}

int attn_fwd_bf16(const void* q, const void* k, const void* v, void* o, float* lse,
                  int B, int H, int N, int d, float scale, int causal, void* stream)
{
    return attn_fwd(q, k, v, o, lse, B, H, N, d, scale, causal, stream, ATTN_FWD_BF16);
}

int attn_fwd_fp8_check_args(const void* q, const void* k, const void* v, const void* o, const float* lse,
                            int B, int H, int N, int d, float scale, int out_dtype)
{
    if (!q || !k || !v || !o || !lse) return ATTN_FWD_ERR_NULL;
    if (B < 1 || H < 1 || N < 1 || (d != 64 && d != 128)) return ATTN_FWD_ERR_SHAPE;
    if (out_dtype != ATTN_FWD_FP16 && out_dtype != ATTN_FWD_BF16) return ATTN_FWD_ERR_SHAPE;
    if (!std::isfinite(scale) || !(scale > 0.0f)) return ATTN_FWD_ERR_SCALE;
    const std::uintptr_t mis = reinterpret_cast<std::uintptr_t>(q) | reinterpret_cast<std::uintptr_t>(k) |
                               reinterpret_cast<std::uintptr_t>(v) | reinterpret_cast<std::uintptr_t>(o) |
                               reinterpret_cast<std::uintptr_t>(lse);
    if (mis & 15u) return ATTN_FWD_ERR_ALIGN;
    // The kernel indexes inside one head with 32-bit byte offsets and numbers its workgroups with an int.
    const unsigned long long head_elems = (unsigned long long)N * (unsigned long long)d;
    if (2ull * head_elems >= (1ull << 31)) return ATTN_FWD_ERR_OVERFLOW;
    const int bm = attn_fp8_launch_tile_param(d, 0);
    const unsigned long long tiles = ((unsigned long long)N + bm - 1) / bm * (unsigned long long)B * (unsigned long long)H;
    if (tiles >= (1ull << 31)) return ATTN_FWD_ERR_OVERFLOW;
    const unsigned long long in_bytes = head_elems * (unsigned long long)B * (unsigned long long)H, out_bytes = 2ull * in_bytes;
    const unsigned long long lse_bytes = 4ull * (unsigned long long)N * (unsigned long long)B * (unsigned long long)H;
    if (overlaps(o, out_bytes, q, in_bytes) || overlaps(o, out_bytes, k, in_bytes) || overlaps(o, out_bytes, v, in_bytes))
        return ATTN_FWD_ERR_ALIAS;
    if (overlaps(lse, lse_bytes, q, in_bytes) || overlaps(lse, lse_bytes, k, in_bytes) || overlaps(lse, lse_bytes, v, in_bytes) ||
        overlaps(lse, lse_bytes, o, out_bytes)) return ATTN_FWD_ERR_ALIAS;
    return ATTN_FWD_OK;
}

int attn_fwd_fp8(const void* q, const void* k, const void* v, void* o, float* lse,
                 int B, int H, int N, int d, float scale, int causal, void* stream, int out_dtype)
{
    const int rc = attn_fwd_fp8_check_args(q, k, v, o, lse, B, H, N, d, scale, out_dtype);
    if (rc != ATTN_FWD_OK) return rc;
    AttnLaunchArgs a{q, k, v, o, lse, B, H, N, d, scale, causal != 0, out_dtype, stream};
    return attn_fp8_launch(a) == 0 ? ATTN_FWD_OK : ATTN_FWD_ERR_LAUNCH;
}

int attn_fwd_fp8_tile_param(int d, int which) { return attn_fp8_launch_tile_param(d, which); }

const char* attn_fwd_strerror(int code)
{
    switch (code) {
        case ATTN_FWD_OK: return "success";
        case ATTN_FWD_ERR_NULL: return "a pointer argument is NULL";
        case ATTN_FWD_ERR_SHAPE: return "unsupported shape or dtype (need B,H,N >= 1, d in {64,128}, dtype in {0,1})";
        case ATTN_FWD_ERR_SCALE: return "scale must be finite and > 0";
        case ATTN_FWD_ERR_ALIGN: return "pointers must be 16-byte aligned";
        case ATTN_FWD_ERR_OVERFLOW: return "problem too large for the kernel's index arithmetic";
        case ATTN_FWD_ERR_LAUNCH: return "HIP refused the kernel launch";
        case ATTN_FWD_ERR_ALIAS: return "o or lse overlaps an input, or each other";
        default: return "unknown error code";
    }
}

int attn_fwd_version(void) { return 100; }

int attn_fwd_tile_param(int d, int causal, int which) { return attn_launch_tile_param(d, causal, which); }

int attn_fwd_tile_schedule(int total, int grid, int block, int round)
{
    if (total < 1 || grid < 1 || grid > total || block < 0 || block >= grid || round < 0) return -2;
    return tile_schedule(total, grid, block, round);
}

int attn_fwd_mfma_probe(float* sink, int workgroups, int iters, int random_operands, int dtype, void* stream)
{
    if (!sink) return ATTN_FWD_ERR_NULL;
    if (workgroups < 1 || workgroups > 65536 || iters < 1 || iters > (1 << 24)) return ATTN_FWD_ERR_SHAPE;
    if (dtype != ATTN_FWD_FP16 && dtype != ATTN_FWD_BF16 && dtype != ATTN_FWD_PROBE_E4M3) return ATTN_FWD_ERR_SHAPE;
    if (reinterpret_cast<std::uintptr_t>(sink) & 3u) return ATTN_FWD_ERR_ALIGN;
    return mfma_probe_launch(sink, workgroups, iters, random_operands != 0, dtype, stream) == 0 ? ATTN_FWD_OK : ATTN_FWD_ERR_LAUNCH;
}

double attn_fwd_mfma_probe_flops(int workgroups, int iters)
{
    if (workgroups < 1 || iters < 1) return 0.0;
    return mfma_probe_flops(workgroups, iters, ATTN_FWD_FP16);
}

double attn_fwd_mfma_probe_flops_of(int workgroups, int iters, int dtype)
{
    if (workgroups < 1 || iters < 1) return 0.0;
    if (dtype != ATTN_FWD_FP16 && dtype != ATTN_FWD_BF16 && dtype != ATTN_FWD_PROBE_E4M3) return 0.0;
    return mfma_probe_flops(workgroups, iters, dtype);
}

int attn_fwd_mfma_probe_sink_floats(int workgroups)
{
    if (workgroups < 1 || workgroups > 65536) return -1;
    return workgroups * mfma_probe_threads();
}

}  // extern "C"
