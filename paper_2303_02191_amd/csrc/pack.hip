// Packing (Section II.B mask semantics: survivors keep their value, the rest are dropped;
// Section IV.D: the tail of a flattened 1x1 tensor is dropped).
//
// pack_live_kernel writes section 0 of the blob: for every group the k surviving weights
// in ascending tap order, and a copy of the group's pattern index.
#include "common.h"
#include "dtypes.h"

namespace rtoss {

template <typename T>
__global__ __launch_bounds__(256) void pack_live_kernel(const T* __restrict__ w, const uint8_t* __restrict__ idx,
                                                        Dict dict, T* __restrict__ live, uint8_t* __restrict__ live_idx,
                                                        int64_t G)
{
    __shared__ uint16_t masks[256];
    masks[threadIdx.x] = (int)threadIdx.x < dict.P ? dict.mask[threadIdx.x] : (uint16_t)0;
    __syncthreads();
    const int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (g >= G) return;
    const uint8_t p = idx[g];
    const unsigned m = masks[p];
    const T* wg = w + g * 9;
    T* out = live + g * dict.k;
    int j = 0;
#pragma unroll
    for (int t = 0; t < 9; ++t)
        if ((m >> t) & 1u) {
            if (j < dict.k) out[j] = wg[t];
            ++j;
        }
    T zero;
    __builtin_memset(&zero, 0, sizeof(T));
    for (; j < dict.k; ++j) out[j] = zero;  // only reached for an index outside the dictionary
    live_idx[g] = p;
}

rtoss_status launch_pack_live(const rtoss_wdesc& d, const void* w, const uint8_t* idx, const Dict& dict,
                              void* live_values, uint8_t* live_idx, int64_t G, hipStream_t s)
{
    if (G == 0) return RTOSS_OK;
    dim3 grid((unsigned)((G + 255) / 256)), block(256);
    switch (d.dt) {
    case RTOSS_F32:
        pack_live_kernel<float><<<grid, block, 0, s>>>((const float*)w, idx, dict, (float*)live_values, live_idx, G);
        break;
    case RTOSS_F16:
        pack_live_kernel<f16_t><<<grid, block, 0, s>>>((const f16_t*)w, idx, dict, (f16_t*)live_values, live_idx, G);
        break;
    case RTOSS_BF16:
        pack_live_kernel<bf16_t><<<grid, block, 0, s>>>((const bf16_t*)w, idx, dict, (bf16_t*)live_values, live_idx, G);
        break;
    }
    return check_hip(hipGetLastError(), "pack launch");
}

}  // namespace rtoss
