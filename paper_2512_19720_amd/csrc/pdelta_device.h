// Device-side helpers shared by the pdelta kernels (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pdelta {

constexpr int kWave = 64;  // CDNA wavefront width

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));
typedef uint32_t uint2v __attribute__((ext_vector_type(2)));

// dtype codes of the C ABI (kept numerically equal to pdelta_dtype in include/pdelta.h)
constexpr int kF16 = 0, kBF16 = 1, kF32 = 2;

// ---- 16-bit storage formats -----------------------------------------------------------------

__device__ __forceinline__ float f16_bits_to_f32(uint32_t h) {
    return (float)__builtin_bit_cast(_Float16, (uint16_t)h);
}
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h) {
    return __builtin_bit_cast(float, h << 16);
}
template <int DT>
__device__ __forceinline__ float bits_to_f32(uint32_t h) {
    return DT == kBF16 ? bf16_bits_to_f32(h) : f16_bits_to_f32(h);
}

// fp32 -> bf16 bits, round to nearest even (finite inputs).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float x) {
    uint32_t u = __builtin_bit_cast(uint32_t, x);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ uint32_t f32_to_f16_bits(float x) {
    return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)x);  // v_cvt_f16_f32, RNE
}

// Store one fp32 result as y_dtype.
template <int YDT>
__device__ __forceinline__ void store_y(void* Y, int64_t idx, float val) {
    if constexpr (YDT == kF32) {
        ((float*)Y)[idx] = val;
    } else if constexpr (YDT == kBF16) {
        ((uint16_t*)Y)[idx] = (uint16_t)f32_to_bf16_bits(val);
    } else {
        ((uint16_t*)Y)[idx] = (uint16_t)f32_to_f16_bits(val);
    }
}

// fp64 -> fp32 with round-to-odd: truncate, then set the last kept bit if anything was lost.
// A later round-to-nearest to a format with <= 22 significant bits then equals a single
// rounding of the fp64 value.  Valid for finite |x| inside fp32's normal range (or zero).
__device__ __forceinline__ float f64_to_f32_round_to_odd(double x) {
    uint64_t u = __builtin_bit_cast(uint64_t, x);
    uint32_t sign = (uint32_t)(u >> 32) & 0x80000000u;
    int32_t e = (int32_t)((u >> 52) & 0x7FF);
    if (e == 0) return __builtin_bit_cast(float, sign);                // +-0 (fp64 subnormals too)
    if (e < 897) return (float)x;                                      // below fp32's normal range
    uint64_t frac = u & 0x000FFFFFFFFFFFFFull;
    uint32_t f32 = (uint32_t)(frac >> 29);                             // top 23 fraction bits
    uint32_t sticky = (frac & 0x1FFFFFFFull) ? 1u : 0u;
    uint32_t bits = sign | ((uint32_t)(e - 1023 + 127) << 23) | f32 | sticky;
    return __builtin_bit_cast(float, bits);
}

// fp64 -> fp16 bits, one rounding to nearest even.  Domain: |x| < 65520 with x a multiple of
// 2^-60 or larger steps (so that the fp32 intermediate is normal or zero).
__device__ __forceinline__ uint32_t f64_to_f16_bits_rne(double x) {
    return f32_to_f16_bits(f64_to_f32_round_to_odd(x));
}
__device__ __forceinline__ uint32_t f64_to_bf16_bits_rne(double x) {
    return f32_to_bf16_bits(f64_to_f32_round_to_odd(x));
}

// Reinterpret one 32-bit register as two fp16 values and back.  Always go through these (a
// by-value scalar): applying __builtin_bit_cast directly to an element of a vector variable
// reads element 0 whatever the index, with this compiler.
__device__ __forceinline__ half2v as_half2(uint32_t u) { return __builtin_bit_cast(half2v, u); }
__device__ __forceinline__ uint32_t as_u32(half2v h) { return __builtin_bit_cast(uint32_t, h); }

// A pointer that a kernel read out of a descriptor in memory is a generic ("flat") pointer to the
// compiler: its loads become flat_load, whose completion counters are shared with LDS, so every
// wait on them is a wait for ALL outstanding loads and a ring of loads in flight degenerates to
// one batch at a time.  Descriptors of this library only ever hold device-global addresses;
// saying so turns the accesses into global_load / global_store with counted waits.
// (The empty asm statement keeps the optimizer from folding the pair of casts away.)
// as_global: for pointers that are uniform across the wavefront (held in scalar registers);
// as_global_per_lane: for pointers that differ between lanes.
template <typename T>
__device__ __forceinline__ T* as_global(T* p) {
    __attribute__((address_space(1))) T* g = (__attribute__((address_space(1))) T*)p;
    asm volatile("" : "+s"(g));
    return (T*)g;
}
template <typename T>
__device__ __forceinline__ T* as_global_per_lane(T* p) {
    __attribute__((address_space(1))) T* g = (__attribute__((address_space(1))) T*)p;
    asm volatile("" : "+v"(g));
    return (T*)g;
}

// ---- wavefront reductions -------------------------------------------------------------------

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, kWave);
    return x;
}
__device__ __forceinline__ unsigned long long wave_sum_u64(unsigned long long x) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, kWave);
    return x;
}
__device__ __forceinline__ double wave_sum_f64(double x) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, kWave);
    return x;
}

}  // namespace pdelta
