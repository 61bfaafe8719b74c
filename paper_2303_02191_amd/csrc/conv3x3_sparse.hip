// 3x3 pattern-sparse convolution on the CDNA4 matrix cores (fp16 / bf16, fp32 accumulate),
// and the packer that writes the weight fragments it streams.
//
// Why 2-of-4 structured sparsity fits pattern pruning (Section IV.B / IV.C): every kernel
// keeps k taps chosen per kernel, so at matrix-tile granularity the zeros are unstructured
// and a dense contraction cannot skip them.  The sparse matrix instruction
// (v_smfmac_f32_16x16x64) accepts a per-row choice of 2 live values in every 4 K-slots.
// For one input channel the 9 taps are split into the 4 corners {0,2,6,8}, the 4 edge
// midpoints {1,3,5,7} and the centre {4}.  Whenever every dictionary pattern has at most
// 2 corners and at most 2 edge midpoints (true for all edge-connected 2- and 3-entry
// patterns: a connected path alternates between the two classes), the corner slots and
// the edge slots of a channel are each one legal 2-of-4 group, and the centre tap is a
// plain dense K-slot.  Per 32 input channels this costs 2+2 sparse steps and 1 dense step
// instead of 9 dense steps.
//
// Instruction operand layout (wave64; r = lane % 16, q = lane / 16):
//   dense  v_mfma_f32_16x16x32:  A lane holds row r, K = 8q .. 8q+7; B lane holds column r,
//          K = 8q .. 8q+7; D lane holds column r, rows 4q .. 4q+3.
//   sparse v_smfmac_f32_16x16x64: A lane holds 8 compressed values of row r in 4 pairs;
//          pair g refers to the 4 B-values (column = any, B lane group 2*(q&1) + (g>>1),
//          B elements 8*(q>>1) + 4*(g&1) .. +3); the two 2-bit fields at bits 4g and 4g+2
//          of the 16-bit index say which of the 4 each compressed value multiplies.
//          ABID selects the low (0) or high (1) half of the index register.
//
// Data flow of one workgroup (256 lanes = 4 waves): output tile = 16*TM output channels x
// (RT x CT) blocks of 4x4 output positions; every wave owns all 16*TM channels and TN of
// the position blocks.  K runs over stages of 32 input channels: the stage's weight
// fragments (one contiguous chunk of the packed blob) and its activation tile with halo
// (channels-last, 32 channels per position, 64-byte position pitch at stride 1 and 80 at stride 2) are copied global ->
// LDS without passing through registers.  B operands are read from LDS as 16-byte vectors
// (8 channels of one tap) and the 4x4 (tap, channel) blocks are transposed in registers
// with byte permutes so that one lane holds, for 4 channels, the 4 taps of a group.
//
// Two kernels share that data flow.  The pipelined one (large layers, stride 1) keeps two
// LDS buffers, one persistent workgroup per compute unit and a hand-placed schedule of
// matrix instructions, LDS reads, permutes and copies.  The single-buffered one (stride 2,
// small layers) is a plain loop nest with small tiles, several workgroups per compute unit.
#include <algorithm>
#include <type_traits>

#include "common.h"
#include "dtypes.h"
#include "epilogue.h"
#include "mma.h"
#include "pack_live.h"
#include "tile3x3.h"

namespace rtoss {

namespace {

// Packed weight fragments: per (stage of 32 input channels, tile of 16 output channels)
//   5 operand fragments of 64 lanes x 16 bytes: corner step 0/1, edge step 0/1, centre
//   then 2 index words per lane: [corner][lane], [edge][lane]; low half = step 0, high = step 1
// (which output channel a row of a tile is: tile_row_channel)
constexpr int kFragBytes = 1024;
constexpr int kTileBytes = 5 * kFragBytes + 2 * 64 * 4;  // 5632
// 16-bit outputs without a fused output stage are stored straight from the accumulators (measured faster
// than the transposition through LDS once a lane's values are 32 contiguous bytes: tile_row_channel)
constexpr bool kDirectEpilogue = true;

__device__ __forceinline__ int tap_of_slot(int group, int f)
{
    // group 0: corners {0,2,6,8}; group 1: edge midpoints {1,3,5,7}
    return group == 0 ? ((f & 1) * 2 + (f >> 1) * 6) : (f == 0 ? 1 : f == 1 ? 3 : f == 2 ? 5 : 7);
}

// Input channel (within a 32-channel stage) that pair g of lane-quarter q refers to in
// sparse step `half`.
__device__ __forceinline__ int stage_channel(int q, int g, int half)
{
    return 8 * (2 * (q & 1) + (g >> 1)) + 4 * half + 2 * (q >> 1) + (g & 1);
}

// Output channel held by row r of channel tile mt.  Within a group of 4 tiles (64 channels) the rows
// are dealt so that the accumulator values one lane holds after the multiplication -- rows
// 4q .. 4q+3 of each of the 4 tiles -- are the 16 consecutive channels 64*(mt/4) + 16q .. +15:
// the epilogues store runs of 16 channels without exchanging data between lanes.
__device__ __forceinline__ int tile_row_channel(int mt, int r)
{
    return 64 * (mt >> 2) + 16 * (r >> 2) + 4 * (mt & 3) + (r & 3);
}
// first of the 4 consecutive channels that quarter q of a lane holds of tile mm (counted from the
// first channel of mm's group of 4 tiles when mm < 4; mm may run over several groups)
__device__ __forceinline__ int tile_quarter_offset(int mm, int q)
{
    return 64 * (mm >> 2) + 16 * q + 4 * (mm & 3);
}

struct SparsePackArgs {
    const void* w;
    const uint8_t* idx;
    char* out;
    int Co, Ci, m_tiles, zero_items;
    int64_t total_items;
    LiveJob job;
};

// One workgroup of one layer (`block` counts from the layer's first block): the first blocks write the
// public section, then comes one block per (stage, channel tile) and last the block of zeros.
// A tile's 16 x 32 kernels (16 rows of 576 contiguous bytes) and their pattern indices are staged in LDS with
// coalesced 16-byte loads; the 5 x 64 fragment pieces are then assembled from LDS.
template <typename T>
__device__ __forceinline__ void pack_sparse3x3_body(const SparsePackArgs& a, const Dict& dict, int block)
{
    const T* __restrict__ w = (const T*)a.w;
    const uint8_t* __restrict__ idx = a.idx;
    char* __restrict__ out = a.out;
    const int Co = a.Co, Ci = a.Ci, m_tiles = a.m_tiles, zero_items = a.zero_items;
    const LiveJob job = a.job;
    __shared__ uint16_t masks[256];
    __shared__ __attribute__((aligned(16))) uint16_t wl[16][32 * 9];  // [row][channel][tap]
    __shared__ __attribute__((aligned(16))) uint8_t il[16][32];       // [row][channel]
    masks[threadIdx.x] = dict.mask[threadIdx.x];
    if (block < job.blocks) {  // the first blocks write the blob's public section
        __syncthreads();
        pack_live_block<T>(w, idx, masks, dict.k, job, block);
        return;
    }
    const int n_tiles = (int)(a.total_items / 320);
    const int tile = block - job.blocks;  // stage * m_tiles + m_tile
    if (tile >= n_tiles) {  // the blocks behind the fragments write the block of zeros, 16 bytes per lane
        const int item = (tile - n_tiles) * 256 + (int)threadIdx.x;
        if (item < zero_items) *(u32x4*)(out + (size_t)n_tiles * kTileBytes + (size_t)item * 16) = u32x4{0, 0, 0, 0};
        return;
    }
    const int mt = tile % m_tiles, cb = tile / m_tiles;
    // ---- stage: 16 rows x 36 chunks of weights, 16 rows x 2 chunks of indices (rows past Co are zeros) ----
    // (rows start at multiples of 576 and 32 bytes from the tensors' first elements; the interface asks for
    // element alignment only, so tensors that do not start on a 16-byte boundary are staged element-wise)
    if (((reinterpret_cast<uintptr_t>(w) | reinterpret_cast<uintptr_t>(idx)) & 15) == 0) {
        for (int c = threadIdx.x; c < 16 * 36; c += 256) {
            const int r = c / 36, k = c % 36;
            const int co = tile_row_channel(mt, r);
            u32x4 v = {0, 0, 0, 0};
            if (co < Co) v = *(const u32x4*)((const char*)w + ((int64_t)co * Ci + 32 * cb) * 18 + k * 16);
            *(u32x4*)((char*)&wl[r][0] + k * 16) = v;
        }
        if (threadIdx.x < 32) {
            const int r = threadIdx.x / 2, k = threadIdx.x % 2;
            const int co = tile_row_channel(mt, r);
            u32x4 v = {0, 0, 0, 0};
            if (co < Co) v = *(const u32x4*)(idx + (int64_t)co * Ci + 32 * cb + k * 16);
            *(u32x4*)(&il[r][k * 16]) = v;
        }
    } else {
        const uint16_t* w16 = (const uint16_t*)w;
        for (int c = threadIdx.x; c < 16 * 288; c += 256) {
            const int r = c / 288, e = c % 288;
            const int co = tile_row_channel(mt, r);
            wl[r][e] = co < Co ? w16[((int64_t)co * Ci + 32 * cb) * 9 + e] : (uint16_t)0;
        }
        for (int c = threadIdx.x; c < 16 * 32; c += 256) {
            const int r = c / 32, e = c % 32;
            const int co = tile_row_channel(mt, r);
            il[r][e] = co < Co ? idx[(int64_t)co * Ci + 32 * cb + e] : (uint8_t)0;
        }
    }
    __syncthreads();
    // ---- assemble: item = (step 0..4, lane); 320 items, the last 64 by the first wave in a second pass ----
    char* tile_out = out + (size_t)tile * kTileBytes;
    for (int item = threadIdx.x; item < 320; item += 256) {
        const int lane = item % 64, step = item / 64;
        const int r = lane % 16, q = lane / 16;
        const bool row_live = tile_row_channel(mt, r) < Co;
        uint16_t vals[8];
        if (step == 4) {  // dense centre tap: K = 8q + j
            for (int j = 0; j < 8; ++j) {
                const int c = 8 * q + j;
                vals[j] = (row_live && ((masks[il[r][c]] >> 4) & 1u)) ? wl[r][c * 9 + 4] : (uint16_t)0;
            }
        } else {
            const int group = step >> 1, half = step & 1;
            unsigned fields = 0;
            for (int g = 0; g < 4; ++g) {
                const int c = stage_channel(q, g, half);
                uint16_t v[2] = {0, 0};
                int f[2] = {0, 1};
                if (row_live) {
                    const unsigned m = masks[il[r][c]];
                    int n = 0;
                    for (int sl = 0; sl < 4; ++sl) {
                        const int t = tap_of_slot(group, sl);
                        if (((m >> t) & 1u) && n < 2) {
                            v[n] = wl[r][c * 9 + t];
                            f[n] = sl;
                            ++n;
                        }
                    }
                    if (n == 1) f[1] = (f[0] + 1) & 3;  // padding value 0 may point anywhere
                }
                vals[2 * g] = v[0];
                vals[2 * g + 1] = v[1];
                fields |= (unsigned)(f[0] | (f[1] << 2)) << (4 * g);
            }
            uint16_t* ip = (uint16_t*)(tile_out + 5 * kFragBytes + (group * 64 + lane) * 4 + half * 2);
            *ip = (uint16_t)fields;
        }
        u32x4 pk;
        pk.x = vals[0] | ((uint32_t)vals[1] << 16);
        pk.y = vals[2] | ((uint32_t)vals[3] << 16);
        pk.z = vals[4] | ((uint32_t)vals[5] << 16);
        pk.w = vals[6] | ((uint32_t)vals[7] << 16);
        *(u32x4*)(tile_out + step * kFragBytes + lane * 16) = pk;
    }
}

template <typename T>
__global__ __launch_bounds__(256) void pack_sparse3x3_kernel(SparsePackArgs a, Dict dict)
{
    pack_sparse3x3_body<T>(a, dict, (int)blockIdx.x);
}

struct SparsePackBatch {
    SparsePackArgs a[kPackBatchMax];
    int first_block[kPackBatchMax + 1];
    int n;
};

template <typename T>
__global__ __launch_bounds__(256) void pack_sparse3x3_batch_kernel(SparsePackBatch b, Dict dict)
{
    const int t = batch_entry(b, (int)blockIdx.x);  // block-uniform
    pack_sparse3x3_body<T>(b.a[t], dict, (int)blockIdx.x - b.first_block[t]);
}

// Channel tiles per stage in the packed section: padded so that every block of 8 tiles is complete.
inline int padded_m_tiles(int Co) { return ((Co + 15) / 16 + 7) / 8 * 8; }
// The section is [fragments][block of zeros]; the zeros feed the copy lanes that fill padding.
inline size_t fragment_bytes(const rtoss_wdesc& d) { return (size_t)(d.Ci / 32) * padded_m_tiles(d.Co) * kTileBytes; }
inline size_t zero_block_bytes(const rtoss_wdesc& d) { return align_up((size_t)2 * d.Ci + 16, 256); }

// When the B operands of the sparse steps are fetched and transposed within a stage of 20 units
// (see the stage loop of conv3x3_sparse_kernel).
template <int TN> struct JobSchedule {
    static constexpr int jobs = 2 * TN;
    static constexpr int load_unit(int q) { return q < TN ? (q - (TN - 3) < -1 ? -1 : q - (TN - 3)) : 6 + (q - TN); }
    static constexpr int perm_count(int u)
    {
        int n = 0;
        for (int q = 0; q < jobs; ++q) n += load_unit(q) + 1 == u;
        return n;
    }
    static constexpr int perm_first(int u)
    {
        for (int q = 0; q < jobs; ++q)
            if (load_unit(q) + 1 == u) return q;
        return 0;
    }
    static constexpr int read_job(int u)
    {
        for (int q = 0; q < jobs; ++q)
            if (load_unit(q) == u) return q;
        return -1;
    }
};

// Single-buffered variant: one LDS buffer, two barriers per stage, plain loop nest scheduled by the
// compiler.  It needs half the LDS of the pipelined kernel below and few registers, so several
// workgroups share a compute unit and hide each other's copy latency and epilogue.  Used for stride 2
// (whose activation tile is too large to keep twice in LDS) and for layers too small for the
// pipelined kernel's 128-channel, 8-stage appetite: TM = 4 covers 64 output channels per workgroup.
template <typename T, typename TO, int S, int TM, int TN, int RT, int CT, bool AHEAD>
__global__ __launch_bounds__(256) void conv3x3_sparse_sb_kernel(const T* __restrict__ x, TO* __restrict__ y,
                                                                const char* __restrict__ wfrag,
                                                                const char* __restrict__ zeros, int H, int W, int Ci,
                                                                int Co, int Ho, int Wo, int m_tiles_total,
                                                                int tiles_c, int tiles_per_image, int co_blocks, int total,
                                                                int work_per_xcd, Epilogue ep)
{
    using G = Geom<S, RT, CT>;
    static_assert(RT * CT == 4 * TN, "four waves share the position blocks of a workgroup");
    constexpr int A_BYTES = TM * kTileBytes;
    constexpr int A_WAVE_COPIES = A_BYTES / 1024;            // 64 lanes x 16 B per copy instruction
    constexpr int A_PER_WAVE = (A_WAVE_COPIES + 3) / 4;
    constexpr int X_CHUNKS = G::x_bytes / 16;                // including the pad chunk of every position
    constexpr int X_PER_WAVE = ((X_CHUNKS + 63) / 64 + 3) / 4;
    static_assert(A_BYTES % 1024 == 0, "weight fragments are whole copy instructions");
    extern __shared__ __attribute__((aligned(16))) char smem[];  // [weights][activations, rounded up to whole copies]
    char* lds_a = smem;
    char* lds_x = smem + A_BYTES;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // Workgroups are dealt to the 8 XCDs in turn.  Work items are numbered with the channel block
    // fastest and each XCD takes a contiguous range, so the workgroups that read the same activation
    // tile (one per channel block) run on one XCD at about the same time and share its L2.
    const int work = (blockIdx.x % 8) * work_per_xcd + blockIdx.x / 8;
    if (work >= total) return;
    const int mt0 = (work % co_blocks) * TM;
    const int tile = (work / co_blocks) % tiles_per_image;
    const int n_img = (work / co_blocks) / tiles_per_image;
    const int tile_r = tile / tiles_c, tile_c = tile % tiles_c;
    const int oh0 = tile_r * G::TH, ow0 = tile_c * G::TW;
    const int ih0 = oh0 * S - 1, iw0 = ow0 * S - 1;
    const int stages = Ci / 32;

    // Copy sources of stage 0.  Every lane copies 16 bytes in every copy instruction; a lane whose LDS
    // slot is zero padding of the tile (or a pad chunk) reads the block of zeros behind the fragments.
    const char* x_ptr[X_PER_WAVE];
#pragma unroll
    for (int k = 0; k < X_PER_WAVE; ++k) {
        const int c = (k * 4 + wave) * 64 + lane;
        const int pos = c / G::kChunks, q = c % G::kChunks;
        const int xr = pos / G::LW, xc = pos % G::LW;
        const int ih = ih0 + xr, iw = iw0 + xc;
        const bool inside = q < 4 && xr < G::IH && xc < G::IW && ih >= 0 && ih < H && iw >= 0 && iw < W;
        // offset in 16-byte chunks: fits 31 bits (checked by the launcher)
        const int off = ((n_img * H + ih) * W + iw) * (Ci >> 3) + q;
        x_ptr[k] = inside ? (const char*)x + (int64_t)off * 16 : zeros;
    }
    const char* a_src = wfrag + (int64_t)mt0 * kTileBytes + lane * 16;
    const int64_t a_stage_stride = (int64_t)m_tiles_total * kTileBytes;

    // ---- per-lane read addresses of the B operand ----
    const int nn = lane & 15, qq = lane >> 4;
    const int pr = nn >> 2, pc = nn & 3;
    int xb[TN];  // byte offset in lds_x of this lane's output position for each of its blocks (tap (0,0))
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int blk = wave * TN + j;
        const int br = blk / CT, bc = blk % CT;
        xb[j] = (((4 * br + pr) * S) * G::LW + (4 * bc + pc) * S) * G::kPos + qq * 16;
    }

    f32x4 acc[TM][TN];
    // (no clearing of the accumulators: the centre step comes first in a stage, and the first stage's
    // writes a * b instead of adding to it)
    auto run_stage = [&](auto first_tag, int stage) {
        constexpr bool FIRST = decltype(first_tag)::value;
        __syncthreads();  // every wave is done reading the previous stage
#pragma unroll
        for (int k = 0; k < A_PER_WAVE; ++k)
            if (k * 4 + wave < A_WAVE_COPIES)  // wave-uniform
                copy16_to_lds(a_src + stage * a_stage_stride + (k * 4 + wave) * 1024, lds_a + (k * 4 + wave) * 1024);
#pragma unroll
        for (int k = 0; k < X_PER_WAVE; ++k) copy16_to_lds(x_ptr[k] + stage * 64, lds_x + (k * 4 + wave) * 1024);
        __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): this wave's copies have landed in LDS
        __syncthreads();                     // ... and everybody's

        // AHEAD: operand reads run ahead of the matrix instructions that use them: the centre step's and
        // the corner group's are issued together, the edge group's behind the centre step.  (The matrix
        // instructions are asm statements that loads are not moved across: source order is issue order.)
        // This hides the LDS latency inside a workgroup; shallow layers over large images, which live on
        // hiding HBM latency across workgroups, do better without it and with the registers it costs.
        u32x4 bc[TN], ac[TM];
        u32x4 rr[2][TN][4], as[2][TM][2];
        int iw2[2][TM];
        auto load_group_x = [&](int group) {
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int f = 0; f < 4; ++f) {
                    const int t = group == 0 ? ((f & 1) * 2 + (f >> 1) * 6) : (2 * f + 1);
                    rr[group][j][f] = *(const u32x4*)(lds_x + xb[j] + ((t / 3) * G::LW + (t % 3)) * G::kPos);
                }
        };
        auto load_group_a = [&](int group, int m) {
            const char* at = lds_a + m * kTileBytes;
            iw2[group][m] = *(const int*)(at + 5 * kFragBytes + (group * 64 + lane) * 4);
            as[group][m][0] = *(const u32x4*)(at + (group * 2 + 0) * kFragBytes + lane * 16);
            as[group][m][1] = *(const u32x4*)(at + (group * 2 + 1) * kFragBytes + lane * 16);
        };
        auto load_group = [&](int group) {
            load_group_x(group);
#pragma unroll
            for (int m = 0; m < TM; ++m) load_group_a(group, m);
        };
        // B operands of both sparse steps of a tap group: element 4*c + f of a step = channel c (of this
        // lane's 4), tap slot f
        u32x8 bf[2][TN];
        auto permute_group = [&](int group) {
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const u32x4(&r)[4] = rr[group][j];
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    const uint32_t s0 = half ? r[0].z : r[0].x, s1 = half ? r[1].z : r[1].x;
                    const uint32_t s2 = half ? r[2].z : r[2].x, s3 = half ? r[3].z : r[3].x;
                    const uint32_t u0 = half ? r[0].w : r[0].y, u1 = half ? r[1].w : r[1].y;
                    const uint32_t u2 = half ? r[2].w : r[2].y, u3 = half ? r[3].w : r[3].y;
                    u32x8 b;
                    b[0] = __builtin_amdgcn_perm(s1, s0, 0x05040100u);  // channel 0: taps 0,1
                    b[1] = __builtin_amdgcn_perm(s3, s2, 0x05040100u);  // channel 0: taps 2,3
                    b[2] = __builtin_amdgcn_perm(s1, s0, 0x07060302u);  // channel 1
                    b[3] = __builtin_amdgcn_perm(s3, s2, 0x07060302u);
                    b[4] = __builtin_amdgcn_perm(u1, u0, 0x05040100u);  // channel 2
                    b[5] = __builtin_amdgcn_perm(u3, u2, 0x05040100u);
                    b[6] = __builtin_amdgcn_perm(u1, u0, 0x07060302u);  // channel 3
                    b[7] = __builtin_amdgcn_perm(u3, u2, 0x07060302u);
                    bf[half][j] = b;
                }
            }
        };
        auto multiply_group = [&](int group, int m) {
#pragma unroll
            for (int j = 0; j < TN; ++j) MatV<T>::template sparse<0>(as[group][m][0], bf[0][j], acc[m][j], iw2[group][m]);
#pragma unroll
            for (int j = 0; j < TN; ++j) MatV<T>::template sparse<1>(as[group][m][1], bf[1][j], acc[m][j], iw2[group][m]);
        };
        auto run_group = [&](int group) {
            permute_group(group);
#pragma unroll
            for (int m = 0; m < TM; ++m) multiply_group(group, m);
        };
        auto load_centre = [&]() {
#pragma unroll
            for (int j = 0; j < TN; ++j) bc[j] = *(const u32x4*)(lds_x + xb[j] + (G::LW + 1) * G::kPos);
#pragma unroll
            for (int m = 0; m < TM; ++m) ac[m] = *(const u32x4*)(lds_a + m * kTileBytes + 4 * kFragBytes + lane * 16);
        };
        auto run_centre = [&]() {  // centre tap: dense step over the 32 channels of the stage
#pragma unroll
            for (int m = 0; m < TM; ++m)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    if constexpr (FIRST) MatV<T>::dense_first(ac[m], bc[j], acc[m][j]);
                    else MatV<T>::dense(ac[m], bc[j], acc[m][j]);
                }
        };
        if constexpr (AHEAD) {
            load_centre();
            load_group(0);
            run_centre();
            load_group(1);
            run_group(0);
            run_group(1);
        } else {  // few operands live at a time: fewer registers, one more workgroup per compute unit
            load_centre();
            run_centre();
#pragma unroll
            for (int group = 0; group < 2; ++group) {
                load_group_x(group);
                permute_group(group);
#pragma unroll
                for (int m = 0; m < TM; ++m) {
                    load_group_a(group, m);
                    multiply_group(group, m);
                }
            }
        }
    };
    run_stage(std::true_type{}, 0);
    for (int stage = 1; stage < stages; ++stage) run_stage(std::false_type{}, stage);

    // the last matrix instructions must have written their accumulators before anything reads them
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    // ---- epilogue: a D lane holds column nn (position) and rows 4*qq .. 4*qq+3 of every channel tile,
    // which tile_row_channel makes 16 consecutive output channels per group of 4 tiles ----
    static_assert(TM % 4 == 0, "whole groups of 4 channel tiles");
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int blk = wave * TN + j;
        const int oh = oh0 + 4 * (blk / CT) + pr, ow = ow0 + 4 * (blk % CT) + pc;
        if (oh >= Ho || ow >= Wo) continue;
        const int64_t pos = ((int64_t)n_img * Ho + oh) * Wo + ow;
        TO* yp = y + pos * ep.ldy;
#pragma unroll
        for (int mg = 0; mg < TM; mg += 4) {
            const int co = 16 * mt0 + tile_quarter_offset(mg, qq);
            if (co >= Co) continue;  // Co is a multiple of 16 and the run of 16 starts at a multiple of 16: all in or all out
            float vv[16];
#pragma unroll
            for (int m = 0; m < 4; ++m)
#pragma unroll
                for (int e = 0; e < 4; ++e) vv[4 * m + e] = acc[mg + m][j][e];
            epi_scale_bias_act<16>(vv, ep, co);
            epi_residual<TO, 16>(vv, ep, pos, co);
            if constexpr (sizeof(TO) == 4) {
#pragma unroll
                for (int g = 0; g < 4; ++g) *(f32x4*)(yp + co + 4 * g) = f32x4{vv[4 * g], vv[4 * g + 1], vv[4 * g + 2], vv[4 * g + 3]};
            } else {
#pragma unroll
                for (int g = 0; g < 2; ++g) {
                    u32x4 o;
                    o.x = pack2_from_f32<TO>(vv[8 * g + 0], vv[8 * g + 1]);
                    o.y = pack2_from_f32<TO>(vv[8 * g + 2], vv[8 * g + 3]);
                    o.z = pack2_from_f32<TO>(vv[8 * g + 4], vv[8 * g + 5]);
                    o.w = pack2_from_f32<TO>(vv[8 * g + 6], vv[8 * g + 7]);
                    *(u32x4*)(yp + co + 8 * g) = o;
                }
            }
        }
    }
}

// FUSED: scale / bias / SiLU / residual in the epilogue.  The plain instantiation (ReLU or nothing) keeps
// its branch-free epilogue; the fused one pays for generality with a few uniform branches per tile.
template <typename T, typename TO, int S, int TM, int TN, int RT, int CT, bool FUSED>
__global__ __launch_bounds__(256, 1) void conv3x3_sparse_kernel(const T* __restrict__ x, TO* __restrict__ y,
                                                                const char* __restrict__ wfrag,
                                                                const char* __restrict__ zeros, int H, int W, int Ci,
                                                                int Co, int Ho, int Wo, int m_tiles_total,
                                                                int tiles_c, int tiles_per_img, int co_blocks,
                                                                int total_work, int work_per_xcd, Epilogue ep)
{
    using G = Geom<S, RT, CT>;
    static_assert(RT * CT == 4 * TN, "four waves share the position blocks of a workgroup");
    static_assert(TN == 4 || TN == 5, "the job schedule below covers 4 or 5 position blocks per wave");
    static_assert(TM == 8, "a stage is 20 units: 5 phases x 4 pairs of channel tiles");
    constexpr int A_BYTES = TM * kTileBytes;
    constexpr int A_WAVE_COPIES = A_BYTES / 1024;              // 64 lanes x 16 B per copy instruction
    constexpr int A_PER_WAVE = (A_WAVE_COPIES + 3) / 4;
    constexpr int X_BYTES = G::x_bytes;
    constexpr int X_CHUNKS = X_BYTES / 16;                     // including the pad chunk of every position
    constexpr int X_WAVE_COPIES = (X_CHUNKS + 63) / 64;
    constexpr int X_PER_WAVE = (X_WAVE_COPIES + 3) / 4;
    constexpr int X_AREA = X_PER_WAVE * 4 * 1024;              // what the copy instructions cover (>= X_BYTES)
    constexpr int REGION = A_BYTES + X_AREA;                   // one pipeline buffer: [weights][activations]
    extern __shared__ __attribute__((aligned(16))) char smem[];  // two regions

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int stages = Ci / 32;
    const int64_t a_stage_stride = (int64_t)m_tiles_total * kTileBytes;

    // Persistent workgroups: one per compute unit, each walking a list of output tiles so that
    // the copies for a tile's first stage overlap the previous tile's last stage and the output
    // stores overlap the next tile's arithmetic.  Workgroups are dealt round-robin to the 8 XCDs
    // (each with its own L2); every XCD gets a contiguous range of work items so that the channel
    // blocks of one spatial tile, and neighbouring tiles, share an L2.
    const int xcd = blockIdx.x % 8, slot_in_xcd = blockIdx.x / 8, slots_per_xcd = gridDim.x / 8;
    const int work_end = min((xcd + 1) * work_per_xcd, total_work);
    int work = xcd * work_per_xcd + slot_in_xcd;
    if (work >= work_end) return;
    // All workgroups run the same code on same-sized tiles, so left alone they reach their
    // epilogues together and the output stores of the whole chip arrive as one burst that the
    // memory system drains while every matrix pipe idles.  Workgroups that own fewer tiles than
    // the busiest one have a tile's worth of slack: they start half a tile late, which moves their
    // store bursts into the others' K loops at no cost to the makespan.
    {
        const int my_tiles = (work_end - work + slots_per_xcd - 1) / slots_per_xcd;
        const int max_tiles = (work_per_xcd + slots_per_xcd - 1) / slots_per_xcd;
        if (my_tiles < max_tiles) {
            const int naps = (stages * 4000 + 8000) / 2 / 8128;  // s_sleep 127 = 127 * 64 cycles
            for (int i = 0; i < naps; ++i) __builtin_amdgcn_s_sleep(127);
        }
    }

    // ---- per-tile state ----
    // Every lane copies 16 bytes in every copy instruction, so the copy code has no branches: a
    // lane whose LDS slot is zero padding of the tile (or an unused pad slot) reads from a block
    // of zeros that the packer appended to the weight fragments (2*Ci + 16 bytes, so that the
    // per-stage advance of 64 bytes stays inside it).
    int n_img, mt0, oh0, ow0;
    const char* x_ptr[X_PER_WAVE];  // per lane and copy slot: source address for stage 0
    auto setup_tile_coords = [&](int w) {
        const int cblk = w % co_blocks;
        const int tile = (w / co_blocks) % tiles_per_img;
        n_img = w / (co_blocks * tiles_per_img);
        mt0 = cblk * TM;
        oh0 = (tile / tiles_c) * G::TH;
        ow0 = (tile % tiles_c) * G::TW;
    };
    auto setup_tile_sources = [&]() {
        const int ih0 = oh0 * S - 1, iw0 = ow0 * S - 1;
#pragma unroll
        for (int k = 0; k < X_PER_WAVE; ++k) {
            const int c = ((k * 4 + wave) * 64 + lane);
            const int pos = c / G::kChunks, q = c % G::kChunks;
            const int pr = pos / G::LW, pc = pos % G::LW;
            const int ih = ih0 + pr, iw = iw0 + pc;
            const bool inside = q < 4 && pr < G::IH && pc < G::IW && ih >= 0 && ih < H && iw >= 0 && iw < W;
            // offset in 16-byte chunks: fits 31 bits (checked by the launcher)
            const int off = ((n_img * H + ih) * W + iw) * (Ci >> 3) + q;
            x_ptr[k] = inside ? (const char*)x + (int64_t)off * 16 : zeros;
        }
    };
    // One copy instruction (64 lanes x 16 bytes) of stage `stage` of the current tile into region
    // `par`: slots 0 .. A_PER_WAVE-1 move weight fragments, the rest move activations.
    constexpr int COPY_SLOTS = A_PER_WAVE + X_PER_WAVE;
    static_assert(COPY_SLOTS <= 20, "two copies per unit in the first ten units of a stage");
    static_assert(A_WAVE_COPIES % 4 == 0, "every wave issues the same number of weight copies");
    auto issue_copy_slot = [&](int slot, int stage, int par) {
        char* region = smem + par * REGION;
        if (slot < A_PER_WAVE) {
            const int kk = slot * 4 + wave;
            const char* asrc = wfrag + (int64_t)mt0 * kTileBytes + lane * 16 + stage * a_stage_stride;
            copy16_to_lds(asrc + kk * 1024, region + kk * 1024);
        } else {
            const int k = slot - A_PER_WAVE;
            const int kk = k * 4 + wave;
            // (the last copy instructions reach past the activation tile into the slack of X_AREA)
            copy16_to_lds(x_ptr[k] + stage * 64, region + A_BYTES + kk * 1024);
        }
    };

    // ---- per-lane read addresses ----
    const int nn = lane & 15, qq = lane >> 4;
    const int pr = nn >> 2, pc = nn & 3;
    // the 4 position blocks of a wave sit at compile-time offsets from the first one
    const int blk0 = wave * TN;
    int xb[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int blk = blk0 + j;
        xb[j] = (((4 * (blk / CT) + pr) * S) * G::LW + (4 * (blk % CT) + pc) * S) * G::kPos + qq * 16;
    }

    f32x4 acc[TM][TN];

    // B operands of the sparse steps need a 4x4 (tap x channel) transpose: a "job" reads the 4 taps of
    // one position block (4 x 16 bytes) and permutes them one pipeline unit later.  Job q < TN = corner
    // taps of block q, job TN + b = edge taps of block b (schedule: JobSchedule).
    using Sched = JobSchedule<TN>;
    constexpr int kJobs = Sched::jobs;
    auto raw_load = [&](const char* X, u32x4 (&rr)[4], int j, int group) {
#pragma unroll
        for (int f = 0; f < 4; ++f) {
            const int t = group == 0 ? ((f & 1) * 2 + (f >> 1) * 6) : (2 * f + 1);
            rr[f] = *(const u32x4*)(X + xb[j] + ((t / 3) * G::LW + (t % 3)) * G::kPos);
        }
    };
    // Operand registers that cross stage boundaries: the reads a stage needs before its first matrix
    // instruction (centre-tap operands of all blocks, weight fragments of unit 0, taps of the jobs
    // permuted in unit 0) are issued from inside the previous stage's last unit.
    u32x4 bc[TN];
    u32x4 rr[kJobs][4];  // every job has its own name; its registers are live from its reads to its permutes
    u32x4 a_nxt[2];
    auto load_stage_prologue = [&](int par) {
        const char* A = smem + par * REGION + lane * 16;
        const char* X = smem + par * REGION + A_BYTES;
#pragma unroll
        for (int j = 0; j < TN; ++j) bc[j] = *(const u32x4*)(X + xb[j] + (G::LW + 1) * G::kPos);
        a_nxt[0] = *(const u32x4*)(A + 4 * kFragBytes);
        a_nxt[1] = *(const u32x4*)(A + kTileBytes + 4 * kFragBytes);
        static_for<kJobs>([&](auto Q) {
            constexpr int q = decltype(Q)::value;
            if constexpr (Sched::load_unit(q) == -1) raw_load(X, rr[q], q % TN, q / TN);
        });
    };

    // (the weight copies need only the tile's channel block: they are under way while the lanes work out
    // their activation sources, ~3 k cycles of address arithmetic)
    setup_tile_coords(work);
#pragma unroll
    for (int slot = 0; slot < A_PER_WAVE; ++slot) issue_copy_slot(slot, 0, 0);
    setup_tile_sources();
#pragma unroll
    for (int slot = A_PER_WAVE; slot < COPY_SLOTS; ++slot) issue_copy_slot(slot, 0, 0);
    __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): this wave's copies have landed in LDS
    __syncthreads();                     // ... and everybody's
    int gpar = 0;     // region that holds the stage about to be multiplied
    load_stage_prologue(0);

  for (;;) {  // tiles
    // output coordinates of the tile being multiplied (the copy state moves on to the next tile early)
    const int t_n = n_img, t_mt0 = mt0, t_oh0 = oh0, t_ow0 = ow0;
    const int next_work = work + slots_per_xcd;
    const bool has_next = next_work < work_end;
    // (no clearing of the accumulators: the first stage's centre step, which visits every one of them
    // first, writes a * b instead of adding to it)
    auto run_stage = [&](auto first_tag, int stage) {
        constexpr bool FIRST = decltype(first_tag)::value;
        // the stage copied while this one is multiplied: the tile's next stage, or the next tile's first
        // (in the very last stage of the last tile there is nothing left to fetch; stage 0 of the
        // same tile is fetched again into the free region, which keeps this code free of branches)
        const bool last_stage = stage + 1 == stages;
        const int copy_stage = last_stage ? 0 : stage + 1;
        if (last_stage && has_next) {
            setup_tile_coords(next_work);
            setup_tile_sources();
        }
        const char* A = smem + gpar * REGION + lane * 16;
        const char* AI = smem + gpar * REGION + 5 * kFragBytes + lane * 4;
        const char* X = smem + gpar * REGION + A_BYTES;

        // One stage = 5 phases (centre, corner step 0/1, edge step 0/1) of TM*TN matrix
        // instructions = 20 units of 2*TN (two channel tiles x TN position blocks).  LDS reads are
        // issued one unit ahead of their use, right after the unit's first matrix instruction,
        // so the wait in front of the next unit's first instruction only covers loads that have
        // had a whole unit to complete; a job's permutes are spread behind the matrix instructions
        // of the unit after its reads.
        //
        // Stage hand-over without a bubble: all of a stage's copies are issued in its first 10 units,
        // and the reads of the last unit's operands are issued in unit 18.  Behind the first matrix
        // instruction of unit 19 the wave therefore waits for its copies and its reads, meets the
        // others at a barrier (the next stage's data is now complete and nobody reads this stage's
        // region any more), and issues the next stage's first reads, which complete under the rest of
        // unit 19.
        // output o (0..15) of a job: dword o%8 of step o/8; element 4*c + f of a step's B operand =
        // channel c (of this lane's 4 in that step), tap slot f
        auto transposed = [&](const u32x4 (&rr)[4], int o) -> uint32_t {
            const int d = o & 7, comp = (o >> 3) * 2 + (d >> 2);
            const uint32_t sel = (d & 2) ? 0x07060302u : 0x05040100u;
            return (d & 1) ? __builtin_amdgcn_perm(rr[3][comp], rr[2][comp], sel)
                           : __builtin_amdgcn_perm(rr[1][comp], rr[0][comp], sel);
        };
        constexpr int UNIT = 2 * TN;  // matrix instructions per unit
        u32x8 bfc[2][TN], bfe[2][TN];
        u32x4 a_cur[2] = {a_nxt[0], a_nxt[1]};
        int i_cur[2] = {0, 0}, i_nxt[2] = {0, 0};

        static_for<20>([&](auto U) {
            constexpr int u = decltype(U)::value;
            constexpr int phase = u / 4, m0 = (u % 4) * 2;
            // jobs permuted in this unit (a contiguous range of job numbers) and the job read in it
            constexpr int perm_first = Sched::perm_first(u), perm_count = Sched::perm_count(u);
            constexpr int job_read = Sched::read_job(u);
            static_for<UNIT>([&](auto I) {
                constexpr int i = decltype(I)::value;
                constexpr int mi = i / TN, j = i % TN, m = m0 + mi;
                if constexpr (phase == 0) {
                    if constexpr (FIRST) Mat<T>::dense_first(a_cur[mi], bc[j], acc[m][j]);
                    else Mat<T>::dense(a_cur[mi], bc[j], acc[m][j]);
                }
                if constexpr (phase == 1) Mat<T>::template sparse<0>(a_cur[mi], bfc[0][j], acc[m][j], i_cur[mi]);
                if constexpr (phase == 2) Mat<T>::template sparse<1>(a_cur[mi], bfc[1][j], acc[m][j], i_cur[mi]);
                if constexpr (phase == 3) Mat<T>::template sparse<0>(a_cur[mi], bfe[0][j], acc[m][j], i_cur[mi]);
                if constexpr (phase == 4) Mat<T>::template sparse<1>(a_cur[mi], bfe[1][j], acc[m][j], i_cur[mi]);
                if constexpr (i == 2 && 2 * u < COPY_SLOTS) issue_copy_slot(2 * u, copy_stage, gpar ^ 1);
                if constexpr (i == 2 + TN && 2 * u + 1 < COPY_SLOTS) issue_copy_slot(2 * u + 1, copy_stage, gpar ^ 1);
                if constexpr (i == 0) {  // issue the next unit's LDS reads behind the first matrix instruction
                    if constexpr (u + 1 < 20) {
                        constexpr int np = (u + 1) / 4, nm0 = ((u + 1) % 4) * 2;
                        constexpr int nstep = np == 0 ? 4 : np - 1;
#pragma unroll
                        for (int t = 0; t < 2; ++t) {
                            a_nxt[t] = *(const u32x4*)(A + (nm0 + t) * kTileBytes + nstep * kFragBytes);
                            if constexpr (np > 0) i_nxt[t] = *(const int*)(AI + (nm0 + t) * kTileBytes + ((np - 1) >> 1) * 256);
                        }
                    }
                    if constexpr (job_read >= 0) raw_load(X, rr[job_read], job_read % TN, job_read / TN);
                    if constexpr (u == 19) {
                        asm volatile("" ::: "memory");
                        __builtin_amdgcn_s_waitcnt(0x0070);  // vmcnt(0) lgkmcnt(0): copies landed, reads of this region done
                        __builtin_amdgcn_s_barrier();
                        asm volatile("" ::: "memory");
                        load_stage_prologue(gpar ^ 1);
                    }
                }
                // this instruction's share of the unit's 16 * perm_count permutes
                constexpr int o_begin = i * 16 * perm_count / UNIT, o_end = (i + 1) * 16 * perm_count / UNIT;
                static_for<o_end - o_begin>([&](auto O) {
                    constexpr int o = o_begin + decltype(O)::value;
                    constexpr int q = perm_first + o / 16, oo = o % 16;
                    const uint32_t v = transposed(rr[q], oo);
                    if constexpr (q < TN) bfc[oo >> 3][q][oo & 7] = v;
                    else bfe[oo >> 3][q - TN][oo & 7] = v;
                });
                __builtin_amdgcn_sched_barrier(0);
            });
            if constexpr (u + 1 < 20) {
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    a_cur[t] = a_nxt[t];
                    i_cur[t] = i_nxt[t];
                }
            }
        });
        gpar ^= 1;
    };
    run_stage(std::true_type{}, 0);
    for (int stage = 1; stage < stages; ++stage) run_stage(std::false_type{}, stage);

    // the last matrix instructions must have written their accumulators before anything reads them
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    // ---- epilogue ----
    // Per lane and group of 4 channel tiles the accumulators hold 16 consecutive output channels of one
    // position (tile_row_channel).  16-bit outputs without a fused output stage are stored directly:
    // 32 contiguous bytes per lane, 128 per position and group.  Otherwise each wave transposes its
    // 64 positions x 16*TM channels through its own slice of the region that was multiplied last
    // (free now; the other region is receiving the next tile's first stage) and writes whole
    // channel rows, 16 bytes per lane; fp32 output goes in two halves of the channel tiles.
    {
        constexpr int EB = (int)sizeof(TO);
        constexpr int HALVES = EB == 4 ? 2 : 1;
        constexpr int TMH = TM / HALVES;
        static_assert(TM % HALVES == 0 && TMH % 4 == 0, "each half is whole groups of 4 channel tiles (tile_row_channel)");
        constexpr int ROW = TMH * 16 * EB + (EB == 2 ? 8 : 16);  // padded row pitch: spreads the banks
        // position blocks staged together: as many as fit when the four waves share one region
        constexpr int JG = (REGION / (4 * 16 * ROW)) < TN ? (REGION / (4 * 16 * ROW)) : TN;
        static_assert(JG >= 1, "epilogue staging must fit in one region");
        char* stage_out = smem + (gpar ^ 1) * REGION + wave * (16 * JG * ROW);
        // lane-derived addresses of the epilogue are recomputed per tile (opaque copy of the lane id)
        // instead of staying live in registers through the K loop
        int lane_e = lane;
        asm volatile("" : "+v"(lane_e));
        const int nn_e = lane_e & 15, qq_e = lane_e >> 4;
        // 64-bit address of the tile's first output element once; everything else is 32-bit
        const int64_t pos_tile = ((int64_t)t_n * Ho + t_oh0) * Wo + t_ow0;  // position number of the tile's first output
        TO* const y_tile = y + pos_tile * ep.ldy;
        const float relu_floor = ep.act == 1 ? 0.f : -__builtin_inff();
        if constexpr (kDirectEpilogue && EB == 2 && !FUSED) {
            // straight from the accumulators: 16 consecutive channels (32 bytes) per lane and group of 4 tiles
            const int pr_e = nn_e >> 2, pc_e = nn_e & 3;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int blk = blk0 + j;
                const int dr = 4 * (blk / CT) + pr_e, dc = 4 * (blk % CT) + pc_e;
                const bool inside = t_oh0 + dr < Ho && t_ow0 + dc < Wo;
                TO* yp = y_tile + (dr * Wo + dc) * ep.ldy + 16 * t_mt0 + 16 * qq_e;
#pragma unroll
                for (int mg = 0; mg < TM; mg += 4) {
                    uint32_t o[8];
#pragma unroll
                    for (int m = 0; m < 4; ++m) {
                        float r[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) asm("v_max_f32 %0, %1, %2" : "=v"(r[e]) : "v"(acc[mg + m][j][e]), "v"(relu_floor));
                        o[2 * m] = pack2_from_f32<TO>(r[0], r[1]);
                        o[2 * m + 1] = pack2_from_f32<TO>(r[2], r[3]);
                    }
                    if (inside && 16 * (t_mt0 + mg) + 16 * qq_e < Co) {
                        *(u32x4*)(yp + 16 * mg) = u32x4{o[0], o[1], o[2], o[3]};
                        *(u32x4*)(yp + 16 * mg + 8) = u32x4{o[4], o[5], o[6], o[7]};
                    }
                }
            }
        } else {
#pragma unroll
        for (int h = 0; h < HALVES; ++h) {
#pragma unroll
          for (int j0 = 0; j0 < TN; j0 += JG) {
            const int jn = j0 + JG <= TN ? JG : TN - j0;  // blocks in this group
#pragma unroll
            for (int jj = 0; jj < jn; ++jj) {
                const int j = j0 + jj;
                f32x4 vals[TMH];
#pragma unroll
                for (int mm = 0; mm < TMH; ++mm) vals[mm] = acc[h * TMH + mm][j];
                // fused ReLU without a branch: max with 0, or with -inf when ReLU is off (one v_max_f32 per
                // value, written as asm so that no NaN-quieting pass is put in front of it)
                if constexpr (FUSED) {
                    // this lane's position in block j and its 4 consecutive channels of every channel tile
                    const int blk_f = blk0 + j;
                    const int dr_f = 4 * (blk_f / CT) + (nn_e >> 2), dc_f = 4 * (blk_f % CT) + (nn_e & 3);
                    const bool inside_f = t_oh0 + dr_f < Ho && t_ow0 + dc_f < Wo;
                    const int64_t pos_f = pos_tile + dr_f * Wo + dc_f;
#pragma unroll
                    for (int mm = 0; mm < TMH; ++mm) {
                        const int co4 = 16 * (t_mt0 + h * TMH) + tile_quarter_offset(mm, qq_e);
                        if (inside_f && co4 < Co) {
                            float vv[4] = {vals[mm].x, vals[mm].y, vals[mm].z, vals[mm].w};
                            epi_scale_bias_act<4>(vv, ep, co4);
                            epi_residual<TO, 4>(vv, ep, pos_f, co4);
                            vals[mm] = f32x4{vv[0], vv[1], vv[2], vv[3]};
                        }
                    }
                } else {
#pragma unroll
                    for (int mm = 0; mm < TMH; ++mm)
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            float r;
                            asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(vals[mm][e]), "v"(relu_floor));
                            vals[mm][e] = r;
                        }
                }
#pragma unroll
                for (int mm = 0; mm < TMH; ++mm) {
                    char* dst = stage_out + (jj * 16 + nn_e) * ROW + tile_quarter_offset(mm, qq_e) * EB;
                    if constexpr (EB == 4) {
                        *(f32x4*)dst = vals[mm];
                    } else {
                        uint2 o;
                        o.x = pack2_from_f32<TO>(vals[mm].x, vals[mm].y);
                        o.y = pack2_from_f32<TO>(vals[mm].z, vals[mm].w);
                        *(uint2*)dst = o;
                    }
                }
            }
            // read back: a row of 16*TMH channels is CH 16-byte chunks; 64 lanes cover 64/CH positions per pass.
            // (A wave's LDS accesses execute in order, so the next group's writes to this slice cannot pass
            // these reads.)
            constexpr int CH = TMH * 16 * EB / 16;
            static_assert(64 % CH == 0, "row chunks must tile the wave");
            constexpr int POS_PER_PASS = 64 / CH;
            static_assert(POS_PER_PASS <= 4 || POS_PER_PASS % 4 == 0, "a pass covers whole rows of a 4x4 block");
            const int passes = (16 * jn) / POS_PER_PASS;
            const int co_first = 16 * (t_mt0 + h * TMH);
            const int sub = lane_e / CH, chunk = lane_e % CH;  // position within the pass, chunk within the row
            const int co = co_first + chunk * (16 / EB);
#pragma unroll
            for (int ps = 0; ps < passes; ++ps) {
                const int p = ps * POS_PER_PASS + sub;
                const int jj = p >> 4, n = p & 15;
                const int blk = blk0 + j0 + jj;
                const int dr = 4 * (blk / CT) + (n >> 2), dc = 4 * (blk % CT) + (n & 3);
                const u32x4 v = *(const u32x4*)(stage_out + p * ROW + chunk * 16);
                if (t_oh0 + dr < Ho && t_ow0 + dc < Wo && co < Co)  // Co is a multiple of 16: a chunk is all in or all out
                    *(u32x4*)(y_tile + (dr * Wo + dc) * ep.ldy + co) = v;
            }
          }
        }
        }
    }
    if (!has_next) break;
    work = next_work;
    // staging slices are read (LDS only): the region may be overwritten by the next copies.  A bare
    // barrier, because __syncthreads() carries a fence that would wait here for this tile's output
    // stores to drain; they drain behind the next tile's first stage instead.  (The direct epilogue
    // does not touch LDS: nothing to wait for.)
    if constexpr (!(kDirectEpilogue && sizeof(TO) == 2 && !FUSED)) {
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0) only
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    }
  }
}

inline bool needs_fused_stage(const ConvParams& c) { return c.ep.scale || c.ep.bias || c.ep.residual || c.ep.act > 1; }

template <typename T, typename TO, int S, int TM, int TN, int RT, int CT, bool FUSED>
rtoss_status launch_variant_f(const rtoss_wdesc& d, const ConvParams& c, const char* wfrag, const void* x, void* y,
                            hipStream_t s)
{
    using G = Geom<S, RT, CT>;
    const int Ho = (c.H + 2 - 3) / S + 1, Wo = (c.W + 2 - 3) / S + 1;
    const int tiles_r = (Ho + G::TH - 1) / G::TH, tiles_c = (Wo + G::TW - 1) / G::TW;
    const int m_tiles_total = padded_m_tiles(d.Co);  // pitch of the packed section
    const int co_blocks = ((d.Co + 15) / 16 + TM - 1) / TM;
    constexpr int x_copies_per_wave = ((G::x_bytes / 16 + 63) / 64 + 3) / 4;
    const size_t smem = 2 * ((size_t)TM * kTileBytes + (size_t)x_copies_per_wave * 4096);
    auto kern = conv3x3_sparse_kernel<T, TO, S, TM, TN, RT, CT, FUSED>;
    static LaunchOnce lds_once;  // per instantiation
    if (rtoss_status st = ensure_dynamic_lds((const void*)kern, smem, lds_once, "conv3x3 shared memory attribute")) return st;
    const int64_t total = (int64_t)tiles_r * tiles_c * co_blocks * c.N;
    if (total > 0x3fffffff) return fail(RTOSS_ESHAPE, "conv: too many tiles");
    if ((int64_t)c.N * c.H * c.W * d.Ci / 8 > 0x7fffffff) return fail(RTOSS_ESHAPE, "conv: input too large for 32-bit chunk offsets");
    const int work_per_xcd = (int)((total + 7) / 8);
    // one workgroup per compute unit (a workgroup owns nearly all of a unit's LDS), at most one per work item
    DeviceInfo dev;
    if (rtoss_status st = current_device(&dev)) return st;
    const int slots_per_xcd = std::max(1, std::min(work_per_xcd, std::max(8, dev.cus) / 8));
    dim3 grid((unsigned)(slots_per_xcd * 8)), block(256);
    const char* zeros = wfrag + fragment_bytes(d);
    kern<<<grid, block, smem, s>>>((const T*)x, (TO*)y, wfrag, zeros, c.H, c.W, d.Ci, d.Co, Ho, Wo, m_tiles_total,
                                   tiles_c, tiles_r * tiles_c, co_blocks, (int)total, work_per_xcd, c.ep);
    return check_hip(hipGetLastError(), "conv3x3 sparse launch");
}

template <typename T, typename TO, int S, int TM, int TN, int RT, int CT>
rtoss_status launch_variant(const rtoss_wdesc& d, const ConvParams& c, const char* wfrag, const void* x, void* y,
                            hipStream_t s)
{
    if constexpr (TN == 4) {  // (the fused output stage is instantiated for the 16x16 tile only)
        if (needs_fused_stage(c)) return launch_variant_f<T, TO, S, TM, TN, RT, CT, true>(d, c, wfrag, x, y, s);
    }
    return launch_variant_f<T, TO, S, TM, TN, RT, CT, false>(d, c, wfrag, x, y, s);
}

template <typename T, typename TO, int S, int TM, int TN, int RT, int CT, bool AHEAD = true>
rtoss_status launch_variant_sb(const rtoss_wdesc& d, const ConvParams& c, const char* wfrag, const void* x, void* y,
                            hipStream_t s)
{
    using G = Geom<S, RT, CT>;
    const int Ho = (c.H + 2 - 3) / S + 1, Wo = (c.W + 2 - 3) / S + 1;
    const int tiles_r = (Ho + G::TH - 1) / G::TH, tiles_c = (Wo + G::TW - 1) / G::TW;
    const int m_tiles_total = padded_m_tiles(d.Co);  // pitch of the packed section
    const int co_blocks = ((d.Co + 15) / 16 + TM - 1) / TM;
    constexpr int x_copies_per_wave = ((G::x_bytes / 16 + 63) / 64 + 3) / 4;
    const size_t smem = (size_t)TM * kTileBytes + (size_t)x_copies_per_wave * 4096;
    auto kern = conv3x3_sparse_sb_kernel<T, TO, S, TM, TN, RT, CT, AHEAD>;
    static LaunchOnce lds_once;  // per instantiation
    if (rtoss_status st = ensure_dynamic_lds((const void*)kern, smem, lds_once, "conv3x3 shared memory attribute")) return st;
    const int64_t total = (int64_t)tiles_r * tiles_c * co_blocks * c.N;
    if (total > 0x3fffffff) return fail(RTOSS_ESHAPE, "conv: too many tiles");
    if ((int64_t)c.N * c.H * c.W * d.Ci / 8 > 0x7fffffff) return fail(RTOSS_ESHAPE, "conv: input too large for 32-bit chunk offsets");
    const int work_per_xcd = (int)((total + 7) / 8);
    dim3 grid((unsigned)(work_per_xcd * 8)), block(256);
    kern<<<grid, block, smem, s>>>((const T*)x, (TO*)y, wfrag, wfrag + fragment_bytes(d), c.H, c.W, d.Ci, d.Co, Ho, Wo,
                                   m_tiles_total, tiles_c, tiles_r * tiles_c, co_blocks, (int)total, work_per_xcd, c.ep);
    return check_hip(hipGetLastError(), "conv3x3 sparse launch");
}

template <typename T, typename TO>
rtoss_status launch_typed(const rtoss_wdesc& d, const ConvParams& c, const char* wfrag, const void* x, void* y,
                          hipStream_t s)
{
    // The fragment section is padded to a multiple of 8 channel tiles, so any TM <= 8 may over-read rows
    // that hold zeros; outputs beyond Co are never stored.
    // Layers with at most 64 output channels, or too few stages to amortise the pipelined kernel's
    // prologue, take the single-buffered kernel with 64 channels per workgroup.
    const bool small = d.Co <= 64 || d.Ci <= 64;
    if (c.stride == 1) {
        // 8x16-position tiles for these: 38 KB of LDS, four workgroups per compute unit.  (Measured: more
        // resident workgroups beat double-buffering inside one, and beat 16x16 tiles, on every such layer.)
        // (up to 64 input channels are one or two stages: nothing to gain inside a workgroup, see AHEAD)
        if (d.Ci <= 64) return launch_variant_sb<T, TO, 1, 4, 2, 2, 4, false>(d, c, wfrag, x, y, s);
        if (small) return launch_variant_sb<T, TO, 1, 4, 2, 2, 4>(d, c, wfrag, x, y, s);
        // ... and so do launches that would leave compute units idle with 128 channels per workgroup
        const int64_t tiles8 = (int64_t)((c.H + 15) / 16) * ((c.W + 15) / 16) * c.N * (((d.Co + 15) / 16 + 7) / 8);
        if (tiles8 < 200) return launch_variant_sb<T, TO, 1, 4, 2, 2, 4>(d, c, wfrag, x, y, s);
        // Two tile shapes: 16x16 positions, or 20 rows x 16 columns (5 position blocks per wave: better
        // reuse of the weight fragments, and for some images fewer rounds over the compute units or less
        // padding).  Cost model: rounds of the busiest workgroup x relative cost of a tile.
        const int Ho = c.H, Wo = c.W;
        const int64_t co_blocks = ((d.Co + 15) / 16 + 7) / 8;
        const int64_t t4 = (int64_t)((Ho + 15) / 16) * ((Wo + 15) / 16) * co_blocks * c.N;
        const int64_t t5 = (int64_t)((Ho + 19) / 20) * ((Wo + 15) / 16) * co_blocks * c.N;
        DeviceInfo dev;
        if (rtoss_status st = current_device(&dev)) return st;
        const int64_t slots = std::max(8, dev.cus) / 8 * 8;  // persistent workgroups of the pipelined kernel
        const double cost4 = (double)((t4 + slots - 1) / slots) * 4.0, cost5 = (double)((t5 + slots - 1) / slots) * 4.85;
        // (with few stages per tile the taller tile's longer prologue and epilogue outweigh the saved round)
        if (cost5 < cost4 && d.Ci >= 128 && !needs_fused_stage(c)) return launch_variant<T, TO, 1, 8, 5, 5, 4>(d, c, wfrag, x, y, s);
        return launch_variant<T, TO, 1, 8, 4, 4, 4>(d, c, wfrag, x, y, s);
    }
    // Stride 2: the input tile of a 16x16 output tile (33x33 positions) nearly fills the LDS by itself.
    // Half-height tiles (8x16 outputs, 17x33 inputs) with 64 channels per workgroup need 72 KB, so two
    // workgroups share a compute unit and overlap each other's copies, and small images pad less.
    // (a single-stage layer is all copy, short multiply, store: quarter-height tiles put three workgroups on a unit)
    if (d.Ci == 32) return launch_variant_sb<T, TO, 2, 4, 1, 1, 4>(d, c, wfrag, x, y, s);
    return launch_variant_sb<T, TO, 2, 4, 2, 2, 4>(d, c, wfrag, x, y, s);
}

}  // namespace

// ---- host-visible entry points of this file ----

bool sparse3x3_dictionary_ok(const Dict& dict)
{
    for (int p = 0; p < dict.P; ++p) {
        const unsigned m = dict.mask[p];
        if (__builtin_popcount(m & 0x145u) > 2 || __builtin_popcount(m & 0x0aau) > 2) return false;
    }
    return true;
}

bool sparse3x3_shape_ok(const rtoss_wdesc& d)
{
    return d.ksize == 3 && (d.dt == RTOSS_F16 || d.dt == RTOSS_BF16) && d.Ci % 32 == 0 && d.Co % 16 == 0;
}

size_t sparse3x3_section_bytes(const rtoss_wdesc& d)
{
    return fragment_bytes(d) + zero_block_bytes(d);
}

static SparsePackArgs sparse_pack_args(const rtoss_wdesc& d, const void* w, const uint8_t* idx, void* section,
                                       void* live_values, uint8_t* live_idx, int* blocks)
{
    SparsePackArgs a;
    a.w = w;
    a.idx = idx;
    a.out = (char*)section;
    a.Co = d.Co;
    a.Ci = d.Ci;
    a.m_tiles = padded_m_tiles(d.Co);
    a.total_items = (int64_t)(d.Ci / 32) * a.m_tiles * 320;
    a.zero_items = (int)(zero_block_bytes(d) / 16);
    a.job = make_live_job(live_values, live_idx, (int64_t)d.Co * d.Ci);
    *blocks = (int)(a.job.blocks + a.total_items / 320 + (a.zero_items + 255) / 256);  // public section, tiles, zeros
    return a;
}

rtoss_status launch_pack_sparse3x3(const rtoss_wdesc& d, const void* w, const uint8_t* idx, const Dict& dict,
                                   void* section, void* live_values, uint8_t* live_idx, hipStream_t s)
{
    int blocks = 0;
    const SparsePackArgs a = sparse_pack_args(d, w, idx, section, live_values, live_idx, &blocks);
    dim3 grid((unsigned)blocks), block(256);
    if (d.dt == RTOSS_F16) pack_sparse3x3_kernel<f16_t><<<grid, block, 0, s>>>(a, dict);
    else pack_sparse3x3_kernel<bf16_t><<<grid, block, 0, s>>>(a, dict);
    return check_hip(hipGetLastError(), "pack sparse3x3 launch");
}

rtoss_status launch_pack_sparse3x3_batch(const PackItem* items, int n, const Dict& dict, hipStream_t s)
{
    for (int base = 0; base < n; base += kPackBatchMax) {
        SparsePackBatch b;
        b.n = std::min(kPackBatchMax, n - base);
        int total = 0;
        for (int i = 0; i < b.n; ++i) {
            const PackItem& it = items[base + i];
            int blocks = 0;
            b.a[i] = sparse_pack_args(it.d, it.w, it.idx, it.section, it.live, it.live_idx, &blocks);
            b.first_block[i] = total;
            total += blocks;
        }
        b.first_block[b.n] = total;
        dim3 grid((unsigned)total), block(256);
        if (items[base].d.dt == RTOSS_F16) pack_sparse3x3_batch_kernel<f16_t><<<grid, block, 0, s>>>(b, dict);
        else pack_sparse3x3_batch_kernel<bf16_t><<<grid, block, 0, s>>>(b, dict);
        if (rtoss_status st = check_hip(hipGetLastError(), "pack sparse3x3 batch launch")) return st;
    }
    return RTOSS_OK;
}

rtoss_status launch_conv3x3_sparse(const rtoss_wdesc& d, const ConvParams& c, const void* section, const void* x,
                                   void* y, hipStream_t s)
{
    const char* wf = (const char*)section;
    const bool f32out = c.out_dt == RTOSS_F32;
    if (d.dt == RTOSS_F16)
        return f32out ? launch_typed<f16_t, float>(d, c, wf, x, y, s) : launch_typed<f16_t, f16_t>(d, c, wf, x, y, s);
    return f32out ? launch_typed<bf16_t, float>(d, c, wf, x, y, s) : launch_typed<bf16_t, bf16_t>(d, c, wf, x, y, s);
}

}  // namespace rtoss
