// Internal seam between the host-side C ABI (gemm_api.cpp) and the kernel (gemm_nt_kernel.hip).
#pragma once

struct GemmLaunchArgs {
    const void* a;   // [M][K]
    const void* b;   // [N][K]
    void* c;         // [M][N]
    int M, N, K;
    int dtype;       // 0 = fp16, 1 = bf16 (for the 8-bit product: the type of c; a and b are E4M3 bytes)
    void* stream;    // hipStream_t
    int config = 0;  // 0 = chosen by K, 1 ... 4 = a fixed kernel configuration (waves per workgroup, paired copies)
};

// Enqueue the kernel for already-validated arguments.  0 on success, -1 if HIP refused the launch.
int gemm_launch(const GemmLaunchArgs& a);

// Rows of C per workgroup (0), columns (1), K tile (2), LDS stages (3), threads per workgroup (4).
int gemm_launch_tile_param(int which);

// The same two calls for the product of 8-bit-float (E4M3) operands (gemm_nt_fp8_kernel.hip).
int gemm_fp8_launch(const GemmLaunchArgs& a);
int gemm_fp8_launch_tile_param(int which);
