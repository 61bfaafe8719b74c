// Pattern selection (Section IV.C, Algorithm 2 scoring loop and best-fit choice, on the
// flat 9-element groups of Section IV.D, Algorithm 3).
//
// Mapping: one workgroup of 256 lanes scores 64 groups.  The 9*64 weights of those groups
// are one contiguous span; the lanes load it element-wise (coalesced), square it in fp64
// and park the squares in LDS.  Every wave holds all 64 groups, one per lane, and scores
// every fourth pattern for them (wave v: patterns v, v+4, ... in ascending order), so the
// pattern and the walk over its live taps are uniform over a wave.  The four (score, index)
// candidates of a group meet in LDS.  Sums run over the live taps in ascending tap order in
// fp64, comparisons are strict, and the merge prefers the lower index on equal scores, so
// the result equals a serial ascending scan bit for bit.
#include <algorithm>

#include "common.h"
#include "dtypes.h"
#include "mma.h"

namespace rtoss {

constexpr int kSelBlock = 256;
constexpr int kSelWaves = kSelBlock / 64;
constexpr int kSelGroupsPerBlock = 64;  // one group per lane of a wave

// One workgroup's share: 64 groups of tensor `w` starting at group g0.
template <typename T>
__device__ __forceinline__ void select_block(const T* __restrict__ w, int64_t G, const Dict& dict, uint8_t* __restrict__ idx,
                                             int64_t g0)
{
    __shared__ double sq[9][kSelGroupsPerBlock];  // tap-major: a wave's 64 reads of one tap are contiguous
    __shared__ double cand_s[kSelWaves][kSelGroupsPerBlock];
    __shared__ int cand_p[kSelWaves][kSelGroupsPerBlock];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t remaining = G - g0;
    const int ngroups = remaining < kSelGroupsPerBlock ? (int)remaining : kSelGroupsPerBlock;

    const T* span = w + g0 * 9;
    // 16-byte loads of whole vectors of the span (a full block is 72 of them for 16-bit weights); the
    // ragged end of a tensor's last block is read element by element
    constexpr int EPV = 16 / (int)sizeof(T);  // elements per vector
    const int n_elems = ngroups * 9;
    static_assert(kSelGroupsPerBlock * 9 <= kSelBlock * EPV, "one vector per lane covers a block");
    {
        const int e0 = tid * EPV;
        // (the interface asks for element alignment only: a span that does not start on a 16-byte boundary
        // takes the element loop as a whole)
        const bool vectors = (reinterpret_cast<uintptr_t>(span) & 15) == 0;
        if (vectors && e0 + EPV <= n_elems) {
            T v[EPV];
            *(u32x4*)v = *(const u32x4*)(span + e0);
#pragma unroll
            for (int i = 0; i < EPV; ++i) {
                const double d = (double)to_f32(v[i]);
                sq[(e0 + i) % 9][(e0 + i) / 9] = d * d;
            }
        } else {
            const int e1 = e0 + EPV < n_elems ? e0 + EPV : n_elems;
            for (int e = e0; e < e1; ++e) {
                const double d = (double)to_f32(span[e]);
                sq[e % 9][e / 9] = d * d;
            }
        }
    }
    __syncthreads();

    // Wave v scores the patterns v, v+4, v+8, ... in ascending order for all 64 groups, lane = group.  The
    // pattern, and so the walk over its live taps (lowest first), is uniform over the wave: per tap one LDS
    // read and one fp64 add per lane.
    double best_s = -1.0;  // below every real score
    int best_p = 0xffff;   // "none yet"
    for (int p = wave; p < dict.P; p += kSelWaves) {
        double s = 0.0;
        for (unsigned m = dict.mask[p]; m != 0; m &= m - 1) s += sq[__builtin_ctz(m)][lane];
        if (s > best_s) { best_s = s; best_p = p; }
    }
    cand_s[wave][lane] = best_s;
    cand_p[wave][lane] = best_p;
    __syncthreads();
    if (wave == 0 && lane < ngroups) {
#pragma unroll
        for (int v = 1; v < kSelWaves; ++v) {
            const double o_s = cand_s[v][lane];
            const int o_p = cand_p[v][lane];
            if (o_s > best_s || (o_s == best_s && o_p < best_p)) { best_s = o_s; best_p = o_p; }
        }
        idx[g0 + lane] = (uint8_t)(best_p == 0xffff ? 0 : best_p);
    }
}

template <typename T>
__global__ __launch_bounds__(kSelBlock) void select_kernel(const T* __restrict__ w, int64_t G, Dict dict,
                                                           uint8_t* __restrict__ idx)
{
    select_block<T>(w, G, dict, idx, (int64_t)blockIdx.x * kSelGroupsPerBlock);
}

// Several tensors in one launch (every layer of a model: the selection of a 1x1 tensor is over its own
// flattening, Section IV.D, so tensors cannot simply be concatenated).  The table travels in the
// launch arguments; a workgroup finds its tensor by a binary search of the table's first-block numbers.
struct SelectBatch {
    const void* w[kSelectBatchMax];
    uint8_t* idx[kSelectBatchMax];
    int64_t G[kSelectBatchMax];
    int first_block[kSelectBatchMax + 1];
    int n;
};

template <typename T>
__global__ __launch_bounds__(kSelBlock) void select_batch_kernel(SelectBatch batch, Dict dict)
{
    const int t = batch_entry(batch, (int)blockIdx.x);  // block-uniform
    select_block<T>((const T*)batch.w[t], batch.G[t], dict, batch.idx[t],
                    (int64_t)((int)blockIdx.x - batch.first_block[t]) * kSelGroupsPerBlock);
}

rtoss_status launch_select_batch(const rtoss_select_item* items, int n, rtoss_dtype dt, const Dict& dict, hipStream_t s)
{
    for (int i = 0; i < n;) {  // i runs on across launches: tensors without a whole group take no table entry
        SelectBatch b;
        b.n = 0;
        int64_t blocks = 0;
        for (; i < n && b.n < kSelectBatchMax; ++i) {
            const int64_t G = items[i].n_elems / 9;
            if (G == 0) continue;
            b.w[b.n] = items[i].w_dev;
            b.idx[b.n] = items[i].idx_dev;
            b.G[b.n] = G;
            b.first_block[b.n] = (int)blocks;
            blocks += (G + kSelGroupsPerBlock - 1) / kSelGroupsPerBlock;
            if (blocks > 0x7fffffffLL) return fail(RTOSS_ESHAPE, "select: too many groups in one batch");
            ++b.n;
        }
        if (b.n == 0) continue;
        b.first_block[b.n] = (int)blocks;
        dim3 grid((unsigned)blocks), block(kSelBlock);
        switch (dt) {
        case RTOSS_F32: select_batch_kernel<float><<<grid, block, 0, s>>>(b, dict); break;
        case RTOSS_F16: select_batch_kernel<f16_t><<<grid, block, 0, s>>>(b, dict); break;
        case RTOSS_BF16: select_batch_kernel<bf16_t><<<grid, block, 0, s>>>(b, dict); break;
        }
        if (rtoss_status st = check_hip(hipGetLastError(), "select batch launch")) return st;
    }
    return RTOSS_OK;
}

rtoss_status launch_select(const void* w, rtoss_dtype dt, int64_t G, const Dict& dict, uint8_t* idx, hipStream_t s)
{
    if (G == 0) return RTOSS_OK;
    const int64_t blocks = (G + kSelGroupsPerBlock - 1) / kSelGroupsPerBlock;
    if (blocks > 0x7fffffffLL) return fail(RTOSS_ESHAPE, "select: too many groups (%lld)", (long long)G);
    dim3 grid((unsigned)blocks), block(kSelBlock);
    switch (dt) {
    case RTOSS_F32: select_kernel<float><<<grid, block, 0, s>>>((const float*)w, G, dict, idx); break;
    case RTOSS_F16: select_kernel<f16_t><<<grid, block, 0, s>>>((const f16_t*)w, G, dict, idx); break;
    case RTOSS_BF16: select_kernel<bf16_t><<<grid, block, 0, s>>>((const bf16_t*)w, G, dict, idx); break;
    }
    return check_hip(hipGetLastError(), "select launch");
}

// Usage count of every pattern (Section IV.B, second narrowing criterion): one byte per group in,
// P counters out.  Each workgroup counts a slice in LDS (integer atomics; the result is independent
// of their order) and adds its non-zero bins to the global counters.
constexpr int kHistBytesPerThread = 16;
constexpr int kHistBlock = 256;
constexpr int kHistChunk = kHistBlock * kHistBytesPerThread;  // indices per workgroup and pass

__global__ __launch_bounds__(kHistBlock) void histogram_kernel(const uint8_t* __restrict__ idx, int64_t G, int P,
                                                               uint32_t* __restrict__ hist)
{
    __shared__ uint32_t bins[256];
    bins[threadIdx.x] = 0;
    __syncthreads();
    for (int64_t base = (int64_t)blockIdx.x * kHistChunk; base < G; base += (int64_t)gridDim.x * kHistChunk) {
        const int64_t g0 = base + (int64_t)threadIdx.x * kHistBytesPerThread;
        // the index tensor comes from an allocator, but its start need not be 16-byte aligned: byte loads
        for (int i = 0; i < kHistBytesPerThread; ++i)
            if (g0 + i < G) {
                const int p = idx[g0 + i];
                if (p < P) atomicAdd(&bins[p], 1u);
            }
    }
    __syncthreads();
    const uint32_t c = bins[threadIdx.x];
    if ((int)threadIdx.x < P && c != 0) atomicAdd(&hist[threadIdx.x], c);
}

rtoss_status launch_histogram(const uint8_t* idx, int64_t G, int P, uint32_t* hist, hipStream_t s)
{
    if (G == 0) return RTOSS_OK;
    const int64_t chunks = (G + kHistChunk - 1) / kHistChunk;
    dim3 grid((unsigned)std::min<int64_t>(chunks, 2048)), block(kHistBlock);
    histogram_kernel<<<grid, block, 0, s>>>(idx, G, P, hist);
    return check_hip(hipGetLastError(), "histogram launch");
}

}  // namespace rtoss
