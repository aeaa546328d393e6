// Internal seam between the host-side C ABI (attn_api.cpp) and the kernels (attn_fwd_kernel.hip).
#pragma once

// Tile configuration compiled into the library.
#ifndef ATTN_CFG_NW
#define ATTN_CFG_NW 8        // waves per workgroup at d = 128: 8 (two wave groups) or 12 (three); d = 64 always 8
#endif
#ifndef ATTN_CFG_MB
#define ATTN_CFG_MB 1        // 32-query blocks per wave at d = 128
#endif
#ifndef ATTN_CFG_MB_D64
#define ATTN_CFG_MB_D64 1    // ... and at d = 64
#endif
#ifndef ATTN_CFG_BN
#define ATTN_CFG_BN 64       // keys per K/V tile
#endif
#ifndef ATTN_CFG_STAGES
#define ATTN_CFG_STAGES 4    // LDS ring depth
#endif

// Schedule of the 16-bit kernel at d = 128: 1 = the in-wave pipeline (attn_fwd_pipe_kernel.hip: every wave
// interleaves the softmax of one tile with the MFMAs of its neighbours), 0 = two wave groups half a
// period apart (attn_fwd_kernel.hip), which also serves d = 64.
#ifndef ATTN_CFG_PIPE
#define ATTN_CFG_PIPE 0
#endif
// Waves per workgroup of the in-wave pipeline: 4 (one per SIMD, 64 query rows each) or 8 (32 rows each).
#ifndef ATTNP_CFG_NW
#define ATTNP_CFG_NW 8
#endif

// Keys per K/V tile of the 8-bit-float kernel, by head dimension.
#ifndef ATTN8_CFG_BN_D128
#define ATTN8_CFG_BN_D128 64
#endif
#ifndef ATTN8_CFG_BN_D64
#define ATTN8_CFG_BN_D64 64
#endif

// LDS ring depth of the 8-bit-float kernel (a stage is 2 x BN x d bytes; 160 KiB per workgroup at most).
#ifndef ATTN8_STAGES
#define ATTN8_STAGES 4
#endif

struct AttnLaunchArgs {
    const void* q;
    const void* k;
    const void* v;
    void* o;
    float* lse;
    int B, H, N, d;
    float scale;
    int causal;
    int dtype;      // 0 = fp16, 1 = bf16 (16-bit kernels: of Q, K, V and O; 8-bit-float kernel: of O)
    void* stream;   // hipStream_t
};

// Enqueue the kernel for already-validated arguments.  0 on success, -1 if HIP refused the launch.
int attn_launch(const AttnLaunchArgs& a);

// Query rows per workgroup (0), keys per tile (1), LDS stages (2), threads per workgroup (3).
int attn_launch_tile_param(int d, int causal, int which);

// The in-wave pipelined kernel (attn_fwd_pipe_kernel.hip), d = 128 only; same contract as attn_launch.
int attn_pipe_launch(const AttnLaunchArgs& a);

// The same for the kernel that takes Q, K, V in E4M3 (attn_fwd_fp8_kernel.hip); a.dtype is the type of O.
int attn_fp8_launch(const AttnLaunchArgs& a);
// Query rows per workgroup (0), keys per tile (1), LDS stages (2), threads per workgroup (3).
int attn_fp8_launch_tile_param(int d, int which);

// Register-only MFMA stream (mfma_probe.hip): `workgroups` workgroups of mfma_probe_threads() threads,
// every wave issuing iters * 8 MFMAs of the given element type; one float per thread is written to sink.
int mfma_probe_launch(float* sink, int workgroups, int iters, int random_operands, int dtype, void* stream);
double mfma_probe_flops(int workgroups, int iters, int dtype);   // dtype 2: E4M3 operands on the 32x32x64 MFMA
int mfma_probe_threads(void);
