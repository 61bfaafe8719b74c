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

// Round to nearest even; gfx950 has a native packed conversion, which the cast selects.
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) { return __builtin_bit_cast(uint16_t, (__bf16)f); }
__device__ __forceinline__ uint16_t f32_to_f16_bits(float f) { return __builtin_bit_cast(uint16_t, (_Float16)f); }

// Two fp32 values -> one dword of two 16-bit values (low half = a).
template <typename T> __device__ __forceinline__ uint32_t pack2_from_f32(float a, float b);
template <> __device__ __forceinline__ uint32_t pack2_from_f32<f16_t>(float a, float b)
{
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    typedef float f2 __attribute__((ext_vector_type(2)));
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f2{a, b}, h2));
}
template <> __device__ __forceinline__ uint32_t pack2_from_f32<bf16_t>(float a, float b)
{
    typedef __bf16 b2 __attribute__((ext_vector_type(2)));
    typedef float f2 __attribute__((ext_vector_type(2)));
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f2{a, b}, b2));
}

template <typename T> __device__ __forceinline__ void store_from_f32(T* p, float v);
template <> __device__ __forceinline__ void store_from_f32<float>(float* p, float v) { *p = v; }
template <> __device__ __forceinline__ void store_from_f32<f16_t>(f16_t* p, float v) { p->bits = f32_to_f16_bits(v); }
template <> __device__ __forceinline__ void store_from_f32<bf16_t>(bf16_t* p, float v) { p->bits = f32_to_bf16_bits(v); }

}  // namespace rtoss
