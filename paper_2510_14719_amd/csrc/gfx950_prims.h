// Device primitives of gfx950 shared by the kernels of this library: vector types, the element-type
// traits (MFMA flavour, fp32 -> 16-bit conversion), direct-to-LDS copies and manual wait counts.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

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
    // acc + lo + hi of a packed pair (the rounded values, as the second contraction sees them)
    static __device__ __forceinline__ float add_pair(unsigned w, float acc) {
        const v2 one = {(_Float16)1.0f, (_Float16)1.0f};
        return __builtin_amdgcn_fdot2(__builtin_bit_cast(v2, w), one, acc, false);
    }
    // The same update for code that sits between MFMAs of its own wave (the dot instructions go through the matrix
    // pipe: measured on MI355X, every v_dot2c there stalls the wave's MFMA stream by a dozen cycles).  fp16: the two
    // unrounded values are added instead; their rounding to fp16 (2^-12 relative, zero mean) is far below what
    // the sum is used for.
    static __device__ __forceinline__ float add_pair_valu(unsigned w, float p0, float p1, float acc) {
        (void)w;
        return acc + p0 + p1;
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
    static __device__ __forceinline__ float add_pair(unsigned w, float acc) {
        const v2 one = {(__bf16)1.0f, (__bf16)1.0f};
        return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(v2, w), one, acc, false);
    }
    // bf16: the ROUNDED values are added (a bf16 is the upper half of its fp32: one shift, one mask).  With 8
    // significant bits the rounding matters: normalising by the sum of the rounded probabilities lets the
    // rounding errors of numerator and denominator cancel on rows that a few keys dominate.
    static __device__ __forceinline__ float add_pair_valu(unsigned w, float p0, float p1, float acc) {
        (void)p0; (void)p1;
        return acc + __builtin_bit_cast(float, w << 16) + __builtin_bit_cast(float, w & 0xffff0000u);
    }
};

// A wave-uniform pointer, moved into scalar registers.
template <typename T> __device__ __forceinline__ T* uniform_ptr(T* p) {
    const unsigned long long a = reinterpret_cast<unsigned long long>(p);
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)a), hi = __builtin_amdgcn_readfirstlane((unsigned)(a >> 32));
    return reinterpret_cast<T*>(((unsigned long long)hi << 32) | lo);
}

// 16 bytes per lane from global memory straight into the LDS: lane L's bytes land at
// lds_addr + 16*L.  The compiler is not told about the transfer (it would otherwise wait for ALL
// outstanding loads before every LDS read); completion is tracked by hand with s_waitcnt vmcnt.
__device__ __forceinline__ void dma16(const void* gbase, unsigned voff, unsigned lds_addr) {
    // (base and LDS address are wave-uniform; the readfirstlanes are free when the compiler already
    // holds them in scalar registers and put them there when it chose vector registers)
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(__builtin_amdgcn_readfirstlane(lds_addr)), "v"(voff), "s"(uniform_ptr(gbase)) : "memory", "m0");
}

template <int N> __device__ __forceinline__ void wait_vmcnt() {
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

}  // namespace
