// Packing (Section II.B mask semantics: survivors keep their value, the rest are dropped;
// Section IV.D: the tail of a flattened 1x1 tensor is dropped).
//
// pack_live_kernel writes section 0 of the blob: for every group the k surviving weights
// in ascending tap order, and a copy of the group's pattern index.
#include "common.h"
#include "dtypes.h"
#include "pack_live.h"

namespace rtoss {

template <typename T>
__global__ __launch_bounds__(256) void pack_live_kernel(const T* __restrict__ w, const uint8_t* __restrict__ idx,
                                                        Dict dict, LiveJob job)
{
    __shared__ uint16_t masks[256];
    masks[threadIdx.x] = dict.mask[threadIdx.x];
    __syncthreads();
    pack_live_block<T>(w, idx, masks, dict.k, job, blockIdx.x);
}

rtoss_status launch_pack_live(const rtoss_wdesc& d, const void* w, const uint8_t* idx, const Dict& dict,
                              void* live_values, uint8_t* live_idx, int64_t G, hipStream_t s)
{
    if (G == 0) return RTOSS_OK;
    const LiveJob job = make_live_job(live_values, live_idx, G);
    dim3 grid((unsigned)job.blocks), block(256);
    switch (d.dt) {
    case RTOSS_F32:
        pack_live_kernel<float><<<grid, block, 0, s>>>((const float*)w, idx, dict, job);
        break;
    case RTOSS_F16:
        pack_live_kernel<f16_t><<<grid, block, 0, s>>>((const f16_t*)w, idx, dict, job);
        break;
    case RTOSS_BF16:
        pack_live_kernel<bf16_t><<<grid, block, 0, s>>>((const bf16_t*)w, idx, dict, job);
        break;
    }
    return check_hip(hipGetLastError(), "pack launch");
}

}  // namespace rtoss
