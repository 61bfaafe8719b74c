// Matrix-core instruction wrappers and the global -> LDS copy shared by the convolution kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <utility>

#include "dtypes.h"

namespace rtoss {

// Compile-time loop: f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>).  The software
// pipelines are written with it so that schedule tables indexed by the loop counter are constants.
template <typename F, int... I> __device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F> __device__ __forceinline__ void static_for(F&& f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x8 __attribute__((ext_vector_type(8)));
typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h16 __attribute__((ext_vector_type(16)));
typedef __bf16 b8 __attribute__((ext_vector_type(8)));
typedef __bf16 b16 __attribute__((ext_vector_type(16)));

// Matrix instructions.  The accumulator is pinned to the accumulation register file ("a"
// constraint) and updated in place, so that the 128 loop-carried accumulator registers of a
// wave never move; everything else (operands, addresses, prefetch) lives in the vector
// registers.  Written as asm because the register class of a builtin's accumulator is the
// allocator's choice and it changes with register pressure.
// Operand hazards: A/B come from LDS reads (waited on by the compiler) or vector ALU results;
// an accumulator is touched again by a matrix instruction no sooner than TN instructions later,
// and is read by other instructions only after the K loop (see the s_nop before the epilogue).
// dense_first: c = a * b through the instruction's constant-zero C operand, the first product of an
// accumulator.  (Clearing accumulators with v_accvgpr_write costs about 18 cycles per register in
// front of the next matrix instruction.)
// MatV is the same with the accumulator in the vector registers: kernels with registers to spare keep
// it there and spare themselves the (equally slow) v_accvgpr_read of the epilogue.
// Hazard the compiler cannot see.  A kernel that needs more than 256 vector registers gets its surplus parked
// in the accumulation registers by the register allocator, which brings a value back with v_accvgpr_read right
// in front of its use.  That move runs through the matrix pipeline, and a matrix instruction that reads its
// result in the next cycles gets the old register contents (seen on the device: wrong sums in exactly the
// accumulator whose operand had been brought back).  The compiler spaces such pairs for instructions it
// knows, not for asm statements.  The build therefore scans the generated code of every kernel for such a
// move close in front of an asm matrix instruction (build.py: check_matrix_hazards) and fails if there is
// one; the kernels are written so that nothing is parked across their matrix loops.  A translation unit
// that cannot be kept clean otherwise may define RTOSS_MFMA_SETTLE, which puts two idle cycles in front of
// every matrix instruction (expensive: a single resident wave per SIMD issues one instruction per 4 cycles,
// so that is 4 cycles per matrix instruction, 15 % on the 256-channel layers).
#ifdef RTOSS_MFMA_SETTLE
#define RTOSS_SETTLE "s_nop 1\n\t"
#else
#define RTOSS_SETTLE ""
#endif
#define RTOSS_MAT_STRUCT(NAME, T, SFX, RW, WO)                                                                        \
    template <> struct NAME<T> {                                                                                      \
        static __device__ __forceinline__ void dense(u32x4 a, u32x4 b, f32x4& c)                                      \
        {                                                                                                             \
            asm volatile(RTOSS_SETTLE "v_mfma_f32_16x16x32_" SFX " %0, %1, %2, %0" : RW(c) : "v"(a), "v"(b));                      \
        }                                                                                                             \
        static __device__ __forceinline__ void dense_first(u32x4 a, u32x4 b, f32x4& c)                                \
        {                                                                                                             \
            asm volatile(RTOSS_SETTLE "v_mfma_f32_16x16x32_" SFX " %0, %1, %2, 0" : WO(c) : "v"(a), "v"(b));                       \
        }                                                                                                             \
        template <int ABID> static __device__ __forceinline__ void sparse(u32x4 a, u32x8 b, f32x4& c, int idx)        \
        {                                                                                                             \
            if (ABID == 0) asm volatile(RTOSS_SETTLE "v_smfmac_f32_16x16x64_" SFX " %0, %1, %2, %3" : RW(c) : "v"(a), "v"(b), "v"(idx)); \
            else asm volatile(RTOSS_SETTLE "v_smfmac_f32_16x16x64_" SFX " %0, %1, %2, %3 abid:1" : RW(c) : "v"(a), "v"(b), "v"(idx));    \
        }                                                                                                             \
    };
template <typename T> struct Mat;
template <typename T> struct MatV;
RTOSS_MAT_STRUCT(Mat, f16_t, "f16", "+a", "=a")
RTOSS_MAT_STRUCT(Mat, bf16_t, "bf16", "+a", "=a")
RTOSS_MAT_STRUCT(MatV, f16_t, "f16", "+v", "=v")
RTOSS_MAT_STRUCT(MatV, bf16_t, "bf16", "+v", "=v")
#undef RTOSS_MAT_STRUCT
#undef RTOSS_SETTLE

// Dense step D = A * B + C over one 16-byte operand per lane, accumulator wherever the compiler keeps it
// (the compiler-scheduled kernels): 32 channels of a 16-bit type in one instruction, or 16 fp32 channels
// in four K = 4 steps, step s on element s of every lane's 16 bytes.
template <typename T> struct Dense16;
template <> struct Dense16<f16_t> {
    static __device__ __forceinline__ f32x4 mma(u32x4 a, u32x4 b, f32x4 c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(h8, a), __builtin_bit_cast(h8, b), c, 0, 0, 0);
    }
};
template <> struct Dense16<bf16_t> {
    static __device__ __forceinline__ f32x4 mma(u32x4 a, u32x4 b, f32x4 c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(b8, a), __builtin_bit_cast(b8, b), c, 0, 0, 0);
    }
};
template <> struct Dense16<float> {
    static __device__ __forceinline__ f32x4 mma(u32x4 a, u32x4 b, f32x4 c)
    {
        const f32x4 af = __builtin_bit_cast(f32x4, a), bf = __builtin_bit_cast(f32x4, b);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(af.x, bf.x, c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(af.y, bf.y, c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(af.z, bf.z, c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(af.w, bf.w, c, 0, 0, 0);
        return c;
    }
};

// One 16-byte global -> LDS copy per lane without passing through registers: lane i of the
// wave writes LDS address lds_wave_base + 16 * i (the base must be wave-uniform).
__device__ __forceinline__ void copy16_to_lds(const void* gsrc, char* lds_wave_base)
{
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gsrc,
                                     (__attribute__((address_space(3))) void*)lds_wave_base, 16, 0, 0);
}

}  // namespace rtoss
