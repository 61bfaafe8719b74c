// The blob's public section 0 (the k survivors of every group in ascending tap order, plus a copy
// of the group's pattern index): this is the mask step W' = W (.) M of Section II.B, and the
// zeroing of a flattened 1x1 tensor's tail (Section IV.D) in the sense that the tail belongs to
// no group.  Shared by the stand-alone packer and by the fragment packers, which do this work in
// their first blocks so that a layer is packed by one launch.
#pragma once
#include "common.h"
#include "dtypes.h"

namespace rtoss {

struct LiveJob {
    void* live;         // [G][k] values
    uint8_t* live_idx;  // [G]
    int64_t G;
    int blocks;         // ceil(G / 256)
};

inline LiveJob make_live_job(void* live, uint8_t* live_idx, int64_t G)
{
    LiveJob j;
    j.live = live;
    j.live_idx = live_idx;
    j.G = G;
    j.blocks = (int)((G + 255) / 256);
    return j;
}

// One block of 256 groups; `masks` is the dictionary in LDS (entries past P are 0).
template <typename T>
__device__ __forceinline__ void pack_live_block(const T* __restrict__ w, const uint8_t* __restrict__ idx,
                                                const uint16_t* masks, int k, const LiveJob& job, int block)
{
    const int64_t g = (int64_t)block * 256 + threadIdx.x;
    if (g >= job.G) return;
    const uint8_t p = idx[g];
    const unsigned m = masks[p];
    const T* wg = w + g * 9;
    T* out = (T*)job.live + g * k;
    int j = 0;
#pragma unroll
    for (int t = 0; t < 9; ++t)
        if ((m >> t) & 1u) {
            if (j < k) out[j] = wg[t];
            ++j;
        }
    T zero;
    __builtin_memset(&zero, 0, sizeof(T));
    for (; j < k; ++j) out[j] = zero;  // only reached for an index outside the dictionary
    job.live_idx[g] = p;
}

}  // namespace rtoss
