// Device-side helpers shared by the gfx950 kernels: 16-bit conversions, wave reductions, vector types.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace qtale {

typedef _Float16 half_t;
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef float float2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));   // 16-byte register value (first-class, unlike a struct)
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));   // 8 bytes of packed 2-bit codes
typedef uint32_t u32x3_t __attribute__((ext_vector_type(3)));   // 12 bytes of packed 3-bit codes (register value)
typedef float float16_t __attribute__((ext_vector_type(16)));

constexpr int kWave = 64;

// ---- 16-bit activation dtype (fp16 or bf16 chosen at run time) --------------------------------
__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) {
    return __uint_as_float(static_cast<uint32_t>(b) << 16);
}
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f) {   // round to nearest even
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<uint16_t>((u >> 16) | 0x40u);  // NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return static_cast<uint16_t>(u >> 16);
}
__device__ __forceinline__ float half_bits_to_float(uint16_t b) {
    return static_cast<float>(__builtin_bit_cast(half_t, b));
}
__device__ __forceinline__ uint16_t float_to_half_bits(float f) {   // round to nearest even, saturating
    f = fminf(fmaxf(f, -65504.0f), 65504.0f);
    return __builtin_bit_cast(uint16_t, static_cast<half_t>(f));
}
template <bool BF16>
__device__ __forceinline__ float act_to_float(uint16_t b) {
    return BF16 ? bf16_bits_to_float(b) : half_bits_to_float(b);
}
template <bool BF16>
__device__ __forceinline__ uint16_t float_to_act(float f) {
    return BF16 ? float_to_bf16_bits(f) : float_to_half_bits(f);
}
__device__ __forceinline__ float act_to_float(uint16_t b, int bf16) {
    return bf16 ? bf16_bits_to_float(b) : half_bits_to_float(b);
}
__device__ __forceinline__ uint16_t float_to_act(float f, int bf16) {
    return bf16 ? float_to_bf16_bits(f) : float_to_half_bits(f);
}

// ---- wave-level reductions (64 lanes) ----------------------------------------------------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

struct alignas(16) U4 { uint32_t x, y, z, w; };
struct alignas(8) U2 { uint32_t x, y; };

}  // namespace qtale
