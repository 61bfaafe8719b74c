// Pattern selection (Section IV.C, Algorithm 2 scoring loop and best-fit choice, on the
// flat 9-element groups of Section IV.D, Algorithm 3).
//
// Mapping: a workgroup is one wave; it scores chunks of 256 groups, four consecutive ones per lane, against
// the whole dictionary.  The 9*256 weights of a chunk are one contiguous span: the lanes load it as 16-byte
// vectors, pass it through LDS so that each lane gets its own 36 weights, square them in fp64 and keep the
// squares in registers.  The pattern is uniform over the wave, so the walk over its taps is scalar control
// flow (one uniform branch per tap position) around plain fp64 adds from registers; with four groups per
// lane the vector unit, not the scalar one, sets the pace (about 150 vector instructions per group for 22
// patterns of 3 taps: 66 adds, 66 for the running best, the rest moves and conversion).  A workgroup can
// take several chunks with all their loads in flight before the first is scored (kSelChunks); measured, one
// chunk per workgroup is faster, because the registers of a second chunk cost more occupancy than the
// overlap returns.  Sums run over the live taps in ascending tap order in fp64 and the patterns are
// scanned in ascending order with a strict comparison, which is the definition's serial scan: the result is
// bit-exact.
#include <algorithm>

#include "common.h"
#include "dtypes.h"
#include "mma.h"

namespace rtoss {

constexpr int kSelBlock = 64;
constexpr int kSelPerLane = 4;
constexpr int kSelGroupsPerChunk = kSelBlock * kSelPerLane;  // 256
constexpr int kSelChunks = 1;                                // chunks per workgroup

template <typename T>
struct SelChunk {
    static constexpr int EPV = 16 / (int)sizeof(T);                     // elements per 16-byte vector
    static constexpr int kSpanElems = kSelGroupsPerChunk * 9;           // 2304
    static constexpr int VPL = (kSpanElems + 64 * EPV - 1) / (64 * EPV);  // vectors per lane: 5 or 9
    const T* span;
    uint8_t* out;  // index of the chunk's first group
    int ngroups;   // 0: no chunk
    bool vectors;
    u32x4 raw[VPL];

    // up to 256 groups of tensor `w` starting at group g0: issues the loads
    __device__ __forceinline__ void load(const T* __restrict__ w, int64_t G, uint8_t* __restrict__ idx, int64_t g0)
    {
        const int lane = threadIdx.x;
        const int64_t remaining = G - g0;
        ngroups = remaining < kSelGroupsPerChunk ? (int)remaining : kSelGroupsPerChunk;
        span = w + g0 * 9;
        out = idx + g0;
        // The interface asks for element alignment only: a span that does not start on a 16-byte boundary
        // takes the element loop as a whole; so does the ragged end of a tensor's last span.
        vectors = (reinterpret_cast<uintptr_t>(span) & 15) == 0;
#pragma unroll
        for (int v = 0; v < VPL; ++v) {
            const int e0 = (v * 64 + lane) * EPV;
            if (vectors && e0 + EPV <= ngroups * 9) raw[v] = *(const u32x4*)(span + e0);
        }
    }

    __device__ __forceinline__ void score(const Dict& dict, T* span_lds) const
    {
        const int lane = threadIdx.x;
        const int n_elems = ngroups * 9;
#pragma unroll
        for (int v = 0; v < VPL; ++v) {
            const int e0 = (v * 64 + lane) * EPV;
            if (vectors && e0 + EPV <= n_elems) {
                *(u32x4*)(span_lds + e0) = raw[v];
            } else {
                const int e1 = e0 + EPV < n_elems ? e0 + EPV : n_elems;
                for (int e = e0; e < e1; ++e) span_lds[e] = span[e];
            }
        }
        __syncthreads();  // (one wave: orders its LDS writes before the reads below)

        // lane's groups 4*lane .. 4*lane+3: 36 consecutive elements.  Lanes past the end of the tensor read
        // whatever LDS holds and their results are dropped.
        double sq[kSelPerLane][9];
        {
            T mine[kSelPerLane * 9];
            constexpr int kBytes = kSelPerLane * 9 * (int)sizeof(T);  // 72 or 144: multiples of 8
            const char* src = reinterpret_cast<const char*>(span_lds) + lane * kBytes;
#pragma unroll
            for (int i = 0; i < kBytes / 8; ++i)
                reinterpret_cast<uint64_t*>(mine)[i] = reinterpret_cast<const uint64_t*>(src)[i];
#pragma unroll
            for (int j = 0; j < kSelPerLane; ++j)
#pragma unroll
                for (int t = 0; t < 9; ++t) {
                    const double d = (double)to_f32(mine[j * 9 + t]);
                    sq[j][t] = d * d;
                }
        }
        __syncthreads();  // the next chunk may overwrite LDS

        double best_s[kSelPerLane];
        int best_p[kSelPerLane];
#pragma unroll
        for (int j = 0; j < kSelPerLane; ++j) { best_s[j] = -1.0; best_p[j] = 0; }  // below every real score
        for (int p2 = 0; 2 * p2 < dict.P; ++p2) {
            uint32_t pair;  // masks 2*p2 and 2*p2+1 in one 32-bit scalar load (there is no 16-bit one)
            __builtin_memcpy(&pair, &dict.mask[2 * p2], 4);
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int p = 2 * p2 + h;
                if (p >= dict.P) break;
                const unsigned m = (pair >> (16 * h)) & 0xffffu;
                double s[kSelPerLane];
#pragma unroll
                for (int j = 0; j < kSelPerLane; ++j) s[j] = 0.0;
#pragma unroll
                for (int t = 0; t < 9; ++t)
                    if (m & (1u << t)) {  // wave-uniform
                        asm volatile("");  // keeps this a branch: as selects it would cost three times the adds
#pragma unroll
                        for (int j = 0; j < kSelPerLane; ++j) s[j] += sq[j][t];
                    }
#pragma unroll
                for (int j = 0; j < kSelPerLane; ++j) {
                    best_p[j] = s[j] > best_s[j] ? p : best_p[j];  // strict: the first of equal scores stays
                    best_s[j] = fmax(best_s[j], s[j]);
                }
            }
        }

        const int first = kSelPerLane * lane;
        uint8_t* o = out + first;
        if (first + kSelPerLane <= ngroups && (reinterpret_cast<uintptr_t>(o) & 3) == 0) {
            *reinterpret_cast<uint32_t*>(o) =
                (uint32_t)best_p[0] | ((uint32_t)best_p[1] << 8) | ((uint32_t)best_p[2] << 16) | ((uint32_t)best_p[3] << 24);
        } else {
#pragma unroll
            for (int j = 0; j < kSelPerLane; ++j)
                if (first + j < ngroups) o[j] = (uint8_t)best_p[j];
        }
    }
};

template <typename T>
__global__ __launch_bounds__(kSelBlock) void select_kernel(const T* __restrict__ w, int64_t G, Dict dict,
                                                           uint8_t* __restrict__ idx)
{
    __shared__ __attribute__((aligned(16))) T span_lds[SelChunk<T>::kSpanElems];
    SelChunk<T> c[kSelChunks];
#pragma unroll
    for (int i = 0; i < kSelChunks; ++i) {
        const int64_t g0 = ((int64_t)blockIdx.x * kSelChunks + i) * kSelGroupsPerChunk;
        c[i].ngroups = 0;
        if (g0 < G) c[i].load(w, G, idx, g0);
    }
#pragma unroll
    for (int i = 0; i < kSelChunks; ++i)
        if (c[i].ngroups > 0) c[i].score(dict, span_lds);  // (workgroup-uniform)
}

// Several tensors in one launch (every layer of a model: the selection of a 1x1 tensor is over its own
// flattening, Section IV.D, so tensors cannot simply be concatenated).  The table travels in the
// launch arguments; chunks are numbered through the tensors in table order.
struct SelectBatch {
    const void* w[kSelectBatchMax];
    uint8_t* idx[kSelectBatchMax];
    int64_t G[kSelectBatchMax];
    int first_chunk[kSelectBatchMax];  // entries past n hold the total
    int n;
    int chunks;
};
static_assert(kSelectBatchMax == 64, "the table lookup below is one entry per lane");

template <typename T>
__global__ __launch_bounds__(kSelBlock) void select_batch_kernel(SelectBatch batch, Dict dict)
{
    __shared__ __attribute__((aligned(16))) T span_lds[SelChunk<T>::kSpanElems];
    // one table entry per lane: a chunk's tensor is the last entry that starts at or before it
    const int my_first = batch.first_chunk[threadIdx.x];
    SelChunk<T> c[kSelChunks];
#pragma unroll
    for (int i = 0; i < kSelChunks; ++i) {
        const int chunk = (int)blockIdx.x * kSelChunks + i;
        c[i].ngroups = 0;
        if (chunk < batch.chunks) {
            const int t = __builtin_popcountll(__ballot(my_first <= chunk)) - 1;
            c[i].load((const T*)batch.w[t], batch.G[t], batch.idx[t],
                      (int64_t)(chunk - batch.first_chunk[t]) * kSelGroupsPerChunk);
        }
    }
#pragma unroll
    for (int i = 0; i < kSelChunks; ++i)
        if (c[i].ngroups > 0) c[i].score(dict, span_lds);
}

rtoss_status launch_select_batch(const rtoss_select_item* items, int n, rtoss_dtype dt, const Dict& dict, hipStream_t s)
{
    for (int i = 0; i < n;) {  // i runs on across launches: tensors without a whole group take no table entry
        SelectBatch b;
        b.n = 0;
        int64_t chunks = 0;
        for (; i < n && b.n < kSelectBatchMax; ++i) {
            const int64_t G = items[i].n_elems / 9;
            if (G == 0) continue;
            b.w[b.n] = items[i].w_dev;
            b.idx[b.n] = items[i].idx_dev;
            b.G[b.n] = G;
            b.first_chunk[b.n] = (int)chunks;
            chunks += (G + kSelGroupsPerChunk - 1) / kSelGroupsPerChunk;
            if (chunks > 0x7fffffffLL) return fail(RTOSS_ESHAPE, "select: too many groups in one batch");
            ++b.n;
        }
        if (b.n == 0) continue;
        for (int t = b.n; t < kSelectBatchMax; ++t) b.first_chunk[t] = (int)chunks;  // never at or before a chunk
        b.chunks = (int)chunks;
        dim3 grid((unsigned)((chunks + kSelChunks - 1) / kSelChunks)), block(kSelBlock);
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
    const int64_t chunks = (G + kSelGroupsPerChunk - 1) / kSelGroupsPerChunk;
    const int64_t blocks = (chunks + kSelChunks - 1) / kSelChunks;
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
