// Measurement aid: a register-only stream of 32x32x16 MFMAs (16-bit operands) or 32x32x64 MFMAs
// (8-bit-float operands) on every SIMD of the chip.
//
// The roofline of the attention kernel is the dense MFMA rate.  The datasheet figure (256 CUs x
// 4 SIMDs x 1024 flop/cycle at 2.4 GHz) assumes the peak clock; under a matrix-core load whose
// operands toggle like real data the power management of the part settles at a lower clock.
// This kernel measures what the matrix cores sustain with no memory traffic and no vector work at
// all: with operands of zeros (no toggling, clock stays at its maximum) and with pseudo-random
// operands (the toggling of real inputs).  The second number is the ceiling any kernel on random
// data can approach; the benchmark reports the attention kernel against both.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "attn_launch.h"

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int PROBE_WAVES = 8;          // two per SIMD, as in the attention kernel
constexpr int PROBE_MFMAS = 8;          // MFMAs per loop iteration and wave

__device__ __forceinline__ unsigned mix(unsigned x) {
    x *= 2654435761u; x ^= x >> 15; x *= 2246822519u; x ^= x >> 13; x *= 3266489917u; x ^= x >> 16;
    return x;
}

// A 16-bit pattern with uniform sign and mantissa and an exponent field that keeps |x| in [2^-3, 2^2):
// every multiplier input toggles, no infinities or NaNs arise.
template <int DTYPE> __device__ __forceinline__ short random_elem(unsigned seed) {
    const unsigned h = mix(seed);
    if (DTYPE == 0) return (short)(((h & 1u) << 15) | ((12u + ((h >> 1) % 5u)) << 10) | ((h >> 8) & 0x3ffu));
    return (short)(((h & 1u) << 15) | ((124u + ((h >> 1) % 5u)) << 7) | ((h >> 8) & 0x7fu));
}

template <int DTYPE>
__global__ __launch_bounds__(PROBE_WAVES * 64)
void mfma_probe_kernel(float* __restrict__ sink, int iters, int random_operands)
{
    s16x8 a[PROBE_MFMAS], b[PROBE_MFMAS];
#pragma unroll
    for (int i = 0; i < PROBE_MFMAS; ++i)
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const unsigned id = ((blockIdx.x * blockDim.x + threadIdx.x) * PROBE_MFMAS + i) * 8 + t;
            a[i][t] = random_operands ? random_elem<DTYPE>(2 * id) : (short)0;
            b[i][t] = random_operands ? random_elem<DTYPE>(2 * id + 1) : (short)0;
        }
    f32x16 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = f32x16(0.f);
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < PROBE_MFMAS; ++i) {
            if (DTYPE == 0)
                acc[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a[i]),
                                                                    __builtin_bit_cast(f16x8, b[(i + 3) % PROBE_MFMAS]), acc[i & 3], 0, 0, 0);
            else
                acc[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[i]),
                                                                     __builtin_bit_cast(bf16x8, b[(i + 3) % PROBE_MFMAS]), acc[i & 3], 0, 0, 0);
        }
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) s += acc[i][j];
    sink[blockIdx.x * blockDim.x + threadIdx.x] = s;   // keeps the accumulators alive
}

// The same stream with E4M3 operands on the 32x32x64 MFMA (dtype 2).  Random bytes have a uniform sign
// and fraction and an exponent field in 5..9 (|x| in [2^-2, 2^3)).
typedef int i32x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ int random_e4m3_word(unsigned seed) {
    int w = 0;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const unsigned h = mix(4 * seed + t);
        w |= (int)((((h & 1u) << 7) | ((5u + ((h >> 1) % 5u)) << 3) | ((h >> 8) & 7u)) << (8 * t));
    }
    return w;
}

__global__ __launch_bounds__(PROBE_WAVES * 64)
void mfma_probe_fp8_kernel(float* __restrict__ sink, int iters, int random_operands)
{
    i32x8 a[PROBE_MFMAS], b[PROBE_MFMAS];
#pragma unroll
    for (int i = 0; i < PROBE_MFMAS; ++i)
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const unsigned id = ((blockIdx.x * blockDim.x + threadIdx.x) * PROBE_MFMAS + i) * 8 + t;
            a[i][t] = random_operands ? random_e4m3_word(2 * id) : 0;
            b[i][t] = random_operands ? random_e4m3_word(2 * id + 1) : 0;
        }
    f32x16 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = f32x16(0.f);
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < PROBE_MFMAS; ++i)
            acc[i & 3] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[i], b[(i + 3) % PROBE_MFMAS], acc[i & 3], 0, 0, 0, 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) s += acc[i][j];
    sink[blockIdx.x * blockDim.x + threadIdx.x] = s;   // keeps the accumulators alive
}

}  // namespace

int mfma_probe_launch(float* sink, int workgroups, int iters, int random_operands, int dtype, void* stream)
{
    const void* kern = dtype == 0 ? reinterpret_cast<const void*>(mfma_probe_kernel<0>)
                     : dtype == 1 ? reinterpret_cast<const void*>(mfma_probe_kernel<1>)
                                  : reinterpret_cast<const void*>(mfma_probe_fp8_kernel);
    void* args[] = {&sink, &iters, &random_operands};
    const hipError_t e = hipLaunchKernel(kern, dim3((unsigned)workgroups), dim3(PROBE_WAVES * 64), args, 0, (hipStream_t)stream);
    return e == hipSuccess ? 0 : -1;
}

double mfma_probe_flops(int workgroups, int iters, int dtype)
{
    return (double)workgroups * PROBE_WAVES * (double)iters * PROBE_MFMAS * (2.0 * 32 * 32 * (dtype == 2 ? 64 : 16));
}

int mfma_probe_threads(void) { return PROBE_WAVES * 64; }
