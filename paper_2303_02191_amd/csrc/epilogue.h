// Fused output stage shared by the convolution kernels:
//     y = act(scale[co] * conv + bias[co]) + residual
// (a folded batch normalisation, the activation and a shortcut connection of the detector
// blocks the pruned layers sit in; Section V reports whole-model inference).  All arithmetic is
// fp32; the result is rounded once when it is stored.
#pragma once
#include "dtypes.h"
#include "mma.h"

namespace rtoss {

struct Epilogue {
    const float* scale;    // [Co] or nullptr (= 1); 16-byte aligned
    const float* bias;     // [Co] or nullptr (= 0); 16-byte aligned
    const void* residual;  // tensor of the output's type and shape, or nullptr
    int act;               // rtoss_act: 0 none, 1 ReLU, 2 SiLU
    // Channels-last tensors: elements from one position's channel 0 to the next position's.  Co for a plain
    // tensor; larger when the convolution writes (or the shortcut reads) a channel slice of a wider buffer,
    // e.g. its part of a concatenation (the slice's first channel is folded into the pointer).
    int ldy;               // of the output
    int ldr;               // of the residual
};

struct ConvParams : rtoss_cdesc {
    Epilogue ep;
};

__device__ __forceinline__ float epi_act(float v, int act)
{
    if (act == 1) return __builtin_fmaxf(v, 0.f);
    if (act == 2) return v / (1.f + __expf(-v));  // v * sigmoid(v)
    return v;
}

// v[0..N) are N consecutive output channels, starting at channel co, of one position (N and co are
// multiples of 4).  Scale, bias and activation; the branches are uniform over the launch.
template <int N> __device__ __forceinline__ void epi_scale_bias_act(float (&v)[N], const Epilogue& ep, int co)
{
    static_assert(N % 4 == 0, "runs of 4 channels");
    if (ep.scale) {
#pragma unroll
        for (int g = 0; g < N / 4; ++g) {
            const f32x4 s = *(const f32x4*)(ep.scale + co + 4 * g);
#pragma unroll
            for (int i = 0; i < 4; ++i) v[4 * g + i] *= s[i];
        }
    }
    if (ep.bias) {
#pragma unroll
        for (int g = 0; g < N / 4; ++g) {
            const f32x4 b = *(const f32x4*)(ep.bias + co + 4 * g);
#pragma unroll
            for (int i = 0; i < 4; ++i) v[4 * g + i] += b[i];
        }
    }
    // (one uniform branch per activation around the whole run, not one per value)
    if (ep.act == 1) {
#pragma unroll
        for (int i = 0; i < N; ++i) v[i] = __builtin_fmaxf(v[i], 0.f);
    } else if (ep.act == 2) {
#pragma unroll
        for (int i = 0; i < N; ++i) v[i] = epi_act(v[i], 2);
    }
}

// Adds the residual's N consecutive channels, starting at channel co, of position number `pos` (n, oh, ow
// flattened) (8-byte aligned runs for 16-bit types, 16-byte aligned for fp32).
template <typename TO, int N> __device__ __forceinline__ void epi_residual(float (&v)[N], const Epilogue& ep, int64_t pos, int co)
{
    static_assert(N % 4 == 0, "runs of 4 elements");
    if (!ep.residual) return;
    const TO* r = (const TO*)ep.residual + pos * ep.ldr + co;
#pragma unroll
    for (int g = 0; g < N / 4; ++g) {
        if constexpr (sizeof(TO) == 4) {
            const f32x4 t = *(const f32x4*)(r + 4 * g);
#pragma unroll
            for (int i = 0; i < 4; ++i) v[4 * g + i] += t[i];
        } else {
            TO t[4];
            *(uint2*)t = *(const uint2*)(r + 4 * g);
#pragma unroll
            for (int i = 0; i < 4; ++i) v[4 * g + i] += to_f32(t[i]);
        }
    }
}

}  // namespace rtoss
