// Device-side element types and exact conversions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rtoss {

struct f16_t { uint16_t bits; };   // IEEE binary16 storage
struct bf16_t { uint16_t bits; };  // bfloat16 storage

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(f16_t v) { return (float)__builtin_bit_cast(_Float16, v.bits); }
__device__ __forceinline__ float to_f32(bf16_t v) { return __builtin_bit_cast(float, (uint32_t)v.bits << 16); }

__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f)
{
    uint32_t u = __builtin_bit_cast(uint32_t, f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);  // quiet NaN
    return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);                  // nearest even
}
__device__ __forceinline__ uint16_t f32_to_f16_bits(float f) { return __builtin_bit_cast(uint16_t, (_Float16)f); }

template <typename T> __device__ __forceinline__ void store_from_f32(T* p, float v);
template <> __device__ __forceinline__ void store_from_f32<float>(float* p, float v) { *p = v; }
template <> __device__ __forceinline__ void store_from_f32<f16_t>(f16_t* p, float v) { p->bits = f32_to_f16_bits(v); }
template <> __device__ __forceinline__ void store_from_f32<bf16_t>(bf16_t* p, float v) { p->bits = f32_to_bf16_bits(v); }

}  // namespace rtoss
