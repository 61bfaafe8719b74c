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
// This file holds the packer and the single-buffered kernel (stride 2, and stride-1 layers with few channels or
// few tiles): a plain loop nest with small tiles, several workgroups per compute unit.  Large stride-1 layers
// take the pipelined kernel of conv3x3_rows.hip, which reads the same packed section.
#include <algorithm>
#include <type_traits>

#include "common.h"
#include "dtypes.h"
#include "epilogue.h"
#include "mma.h"
#include "pack_live.h"
#include "sparse_frag.h"
#include "tile3x3.h"

namespace rtoss {

namespace {

// Input channel (within a 32-channel stage) that pair g of lane-quarter q refers to in
// sparse step `half`.
__device__ __forceinline__ int stage_channel(int q, int g, int half)
{
    return 8 * (2 * (q & 1) + (g >> 1)) + 4 * half + 2 * (q >> 1) + (g & 1);
}

constexpr int kMaxTapGroups = 3;  // tap groups of a layout (TapLayout::tap)

struct SparsePackArgs {
    const void* w;
    const uint8_t* idx;
    char* out;
    int Co, Ci, m_tiles, zero_items;
    int64_t total_items;  // 64 * fragments per tile * tiles
    LiveJob job;
};

// One workgroup of one layer (`block` counts from the layer's first block): the first blocks write the
// public section, then comes one block per (stage, channel tile) and last the block of zeros.
// A tile's 16 x 32 kernels (16 rows of 576 contiguous bytes) and their pattern indices are staged in LDS with
// coalesced 16-byte loads; the fragment pieces (64 per fragment) are then assembled from LDS.
template <typename T>
__device__ __forceinline__ void pack_sparse3x3_body(const SparsePackArgs& a, const TapLayout& lay, const Dict& dict, int block)
{
    const T* __restrict__ w = (const T*)a.w;
    const uint8_t* __restrict__ idx = a.idx;
    char* __restrict__ out = a.out;
    const int Co = a.Co, Ci = a.Ci, m_tiles = a.m_tiles, zero_items = a.zero_items;
    const LiveJob job = a.job;
    const int frags = layout_fragments(lay), tile_bytes = layout_tile_bytes(lay);
    __shared__ uint16_t masks[256];
    __shared__ __attribute__((aligned(16))) uint16_t wl[16][32 * 9];  // [row][channel][tap]
    __shared__ __attribute__((aligned(16))) uint8_t il[16][32];       // [row][channel]
    __shared__ uint16_t slots[256 * kMaxTapGroups];
    constexpr unsigned kNoTaps = 15u | (15u << 4) | (0u << 8) | (1u << 10);  // a row past Co: zeros, slots 0 and 1
    masks[threadIdx.x] = dict.mask[threadIdx.x];
    if (block < job.blocks) {  // the first blocks write the blob's public section
        __syncthreads();
        pack_live_block<T>(w, idx, masks, dict.k, job, block);
        return;
    }
    const int n_tiles = (int)(a.total_items / (64 * frags));
    const int tile = block - job.blocks;  // stage * m_tiles + m_tile
    if (tile >= n_tiles) {  // the blocks behind the fragments write the block of zeros, 16 bytes per lane
        const int item = (tile - n_tiles) * 256 + (int)threadIdx.x;
        if (item < zero_items) *(u32x4*)(out + (size_t)n_tiles * tile_bytes + (size_t)item * 16) = u32x4{0, 0, 0, 0};
        return;
    }
    const int mt = tile % m_tiles, cb = tile / m_tiles;
    // slots[p][group]: taps of pattern p's first and second live tap in the group (bits 0-3, 4-7; 15: none) and the
    // slots they take (bits 8-9, 10-11; a missing second value points at the slot after the first, a group without
    // live taps at slots 0 and 1: padding values of 0 may point anywhere, as long as the two differ)
    for (int e = threadIdx.x; e < dict.P * kMaxTapGroups; e += 256) {
        const int p = e / kMaxTapGroups, group = e % kMaxTapGroups;
        unsigned tp[2] = {15u, 15u}, f[2] = {0u, 1u};
        if (group < lay.groups) {
            const unsigned m = dict.mask[p];
            int n = 0;
            for (int sl = 0; sl < 4; ++sl) {
                const int tt = lay.tap[group][sl];
                if (tt >= 0 && ((m >> tt) & 1u) && n < 2) {
                    tp[n] = (unsigned)tt;
                    f[n] = (unsigned)sl;
                    ++n;
                }
            }
            if (n == 1) f[1] = (f[0] + 1) & 3;
        }
        slots[e] = (uint16_t)(tp[0] | (tp[1] << 4) | (f[0] << 8) | (f[1] << 10));
    }
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
    // ---- assemble: item = (fragment, lane).  What a pattern puts into a tap group -- which of the group's four slots
    // its (at most two) live taps take, and which taps those are -- comes from the table built above, so the walk over
    // the 4 x 4 (channel, slot) pairs of an item has no data-dependent branch. ----
    char* tile_out = out + (size_t)tile * tile_bytes;
    for (int item = threadIdx.x; item < 64 * frags; item += 256) {
        const int lane = item % 64, step = item / 64;  // (step is uniform over a wave)
        const int r = lane % 16, q = lane / 16;
        const bool row_live = tile_row_channel(mt, r) < Co;
        uint16_t vals[8];
        if (step == 2 * lay.groups) {  // dense centre tap: K = 8q + j
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int c = 8 * q + j;
                const uint16_t v = wl[r][c * 9 + 4];
                vals[j] = (row_live && ((masks[il[r][c]] >> 4) & 1u)) ? v : (uint16_t)0;
            }
        } else {
            const int group = step >> 1, half = step & 1;
            unsigned fields = 0;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int c = stage_channel(q, g, half);
                const unsigned e = row_live ? slots[il[r][c] * kMaxTapGroups + group] : kNoTaps;
                const unsigned t0 = e & 15u, t1 = (e >> 4) & 15u;  // taps of the two values (15: none)
                const uint16_t v0 = wl[r][c * 9 + (t0 < 9 ? t0 : 0)], v1 = wl[r][c * 9 + (t1 < 9 ? t1 : 0)];
                vals[2 * g] = t0 < 9 ? v0 : (uint16_t)0;
                vals[2 * g + 1] = t1 < 9 ? v1 : (uint16_t)0;
                fields |= ((e >> 8) & 15u) << (4 * g);  // slot of the first value | slot of the second << 2
            }
            uint16_t* ip = (uint16_t*)(tile_out + frags * kFragBytes + (group * 64 + lane) * 4 + half * 2);
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
__global__ __launch_bounds__(256) void pack_sparse3x3_kernel(SparsePackArgs a, TapLayout lay, Dict dict)
{
    pack_sparse3x3_body<T>(a, lay, dict, (int)blockIdx.x);
}

struct SparsePackBatch {
    SparsePackArgs a[kPackBatchMax];
    int first_block[kPackBatchMax + 1];
    int n;
    TapLayout layout;  // (one dictionary per batch: one layout)
};

template <typename T>
__global__ __launch_bounds__(256) void pack_sparse3x3_batch_kernel(SparsePackBatch b, Dict dict)
{
    const int t = batch_entry(b, (int)blockIdx.x);  // block-uniform
    pack_sparse3x3_body<T>(b.a[t], b.layout, dict, (int)blockIdx.x - b.first_block[t]);
}

// Single-buffered variant: one LDS buffer, two barriers per stage, plain loop nest scheduled by the
// compiler.  It needs half the LDS of the pipelined kernel below and few registers, so several
// workgroups share a compute unit and hide each other's copy latency and epilogue.  Used for stride 2
// (whose activation tile is too large to keep twice in LDS) and for layers too small for the
// pipelined kernel's 128-channel, 8-stage appetite: TM = 4 covers 64 output channels per workgroup.
// LAY: tap layout (sparse_frag.h).  Layout 1 (4-entry dictionaries) has three tap groups and no dense centre
// step; it always takes the one-group-at-a-time schedule.
// DB: two LDS buffers; the copies of the next stage are issued right after the barrier that opens a stage and land
// while it is multiplied (one barrier per stage).  For deep stride-1 layers, whose schedule with operand reads ahead
// is held to two workgroups per compute unit by its registers anyway: two buffers of 38 KB each still fit twice.
template <typename T, typename TO, int S, int TM, int TN, int RT, int CT, bool AHEAD, int LAY = 0, bool DB = false>
__global__ __launch_bounds__(256) void conv3x3_sparse_sb_kernel(const T* __restrict__ x, TO* __restrict__ y,
                                                                const char* __restrict__ wfrag,
                                                                const char* __restrict__ zeros, int H, int W, int Ci,
                                                                int Co, int Ho, int Wo, int m_tiles_total,
                                                                int tiles_c, int tiles_per_image, int co_blocks, int total,
                                                                int work_per_xcd, Epilogue ep)
{
    using G = Geom<S, RT, CT>;
    static_assert(RT * CT == 4 * TN, "four waves share the position blocks of a workgroup");
    constexpr TapLayout LY = kLayouts[LAY];
    constexpr int NG = LY.groups, FR = layout_fragments(LY), TILE = layout_tile_bytes(LY);
    constexpr int A_BYTES = TM * TILE;
    constexpr int A_WAVE_COPIES = A_BYTES / 1024;            // 64 lanes x 16 B per copy instruction
    constexpr int A_PER_WAVE = (A_WAVE_COPIES + 3) / 4;
    constexpr int X_CHUNKS = G::x_bytes / 16;                // including the pad chunk of every position
    constexpr int X_PER_WAVE = ((X_CHUNKS + 63) / 64 + 3) / 4;
    static_assert(A_BYTES % 1024 == 0, "weight fragments are whole copy instructions");
    extern __shared__ __attribute__((aligned(16))) char smem[];  // [weights][activations, rounded up to whole copies] (x2 with DB)
    constexpr int BUF = A_BYTES + X_PER_WAVE * 4096;
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

    const char* a_src = wfrag + (int64_t)mt0 * TILE + lane * 16;
    const int64_t a_stage_stride = (int64_t)m_tiles_total * TILE;
    auto issue_weight_copies = [&](int stage, char* buf) {
#pragma unroll
        for (int k = 0; k < A_PER_WAVE; ++k)
            if (k * 4 + wave < A_WAVE_COPIES)  // wave-uniform
                copy16_to_lds(a_src + stage * a_stage_stride + (k * 4 + wave) * 1024, buf + (k * 4 + wave) * 1024);
    };
    // (the weight fragments of stage 0 need only the channel block: they are under way while the lanes work out
    // their activation sources)
    issue_weight_copies(0, smem);

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
    auto issue_copies = [&](int stage, char* buf, bool with_weights) {
        if (with_weights) issue_weight_copies(stage, buf);
#pragma unroll
        for (int k = 0; k < X_PER_WAVE; ++k) copy16_to_lds(x_ptr[k] + stage * 64, buf + A_BYTES + (k * 4 + wave) * 1024);
    };
    if constexpr (DB) issue_copies(0, smem, false);
    auto run_stage = [&](auto first_tag, int stage) {
        constexpr bool FIRST = decltype(first_tag)::value;
        if constexpr (DB) {
            __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): this wave's copies of this stage have landed in LDS
            __syncthreads();                     // ... and everybody's; and every wave is done reading the other buffer
            const int par = stage & 1;
            if (stage + 1 < stages) issue_copies(stage + 1, smem + (par ^ 1) * BUF, true);
            lds_a = smem + par * BUF;
            lds_x = lds_a + A_BYTES;
        } else {
            __syncthreads();  // every wave is done reading the previous stage
            issue_copies(stage, smem, !FIRST);  // (stage 0's weight fragments are already under way)
            __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): this wave's copies have landed in LDS
            __syncthreads();                     // ... and everybody's
        }

        // AHEAD: operand reads run ahead of the matrix instructions that use them: the centre step's and
        // the corner group's are issued together, the edge group's behind the centre step.  (The matrix
        // instructions are asm statements that loads are not moved across: source order is issue order.)
        // This hides the LDS latency inside a workgroup; shallow layers over large images, which live on
        // hiding HBM latency across workgroups, do better without it and with the registers it costs.
        u32x4 bc[TN], ac[TM];
        u32x4 rr[NG][TN][4], as[NG][TM][2];
        int iw2[NG][TM];
        auto load_group_x = [&](int group) {
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int f = 0; f < 4; ++f) {
                    // (an empty slot carries weight 0: it reads the group's first tap, any finite value does)
                    const int t = LY.tap[group][f] >= 0 ? LY.tap[group][f] : LY.tap[group][0];
                    rr[group][j][f] = *(const u32x4*)(lds_x + xb[j] + ((t / 3) * G::LW + (t % 3)) * G::kPos);
                }
        };
        auto load_group_a = [&](int group, int m) {
            const char* at = lds_a + m * TILE;
            iw2[group][m] = *(const int*)(at + FR * kFragBytes + (group * 64 + lane) * 4);
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
            for (int m = 0; m < TM; ++m) ac[m] = *(const u32x4*)(lds_a + m * TILE + 2 * NG * kFragBytes + lane * 16);
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
        if constexpr (AHEAD && LAY == 0) {
            load_centre();
            load_group(0);
            run_centre();
            load_group(1);
            run_group(0);
            run_group(1);
        } else {  // few operands live at a time: fewer registers, one more workgroup per compute unit
            if constexpr (LY.centre) {
                load_centre();
                run_centre();
            } else if constexpr (FIRST) {  // (no dense step that could write the first product: clear)
#pragma unroll
                for (int m = 0; m < TM; ++m)
#pragma unroll
                    for (int j = 0; j < TN; ++j) acc[m][j] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
            for (int group = 0; group < NG; ++group) {
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

template <typename T, typename TO, int S, int TM, int TN, int RT, int CT, bool AHEAD = true, int LAY = 0, bool DB = false>
rtoss_status launch_variant_sb(const rtoss_wdesc& d, const ConvParams& c, const char* wfrag, const void* x, void* y,
                            hipStream_t s)
{
    using G = Geom<S, RT, CT>;
    const int Ho = (c.H + 2 - 3) / S + 1, Wo = (c.W + 2 - 3) / S + 1;
    const int tiles_r = (Ho + G::TH - 1) / G::TH, tiles_c = (Wo + G::TW - 1) / G::TW;
    const int m_tiles_total = padded_m_tiles(d.Co);  // pitch of the packed section
    const int co_blocks = ((d.Co + 15) / 16 + TM - 1) / TM;
    constexpr int x_copies_per_wave = ((G::x_bytes / 16 + 63) / 64 + 3) / 4;
    const size_t smem = (DB ? 2 : 1) * ((size_t)TM * layout_tile_bytes(kLayouts[LAY]) + (size_t)x_copies_per_wave * 4096);
    auto kern = conv3x3_sparse_sb_kernel<T, TO, S, TM, TN, RT, CT, AHEAD, LAY, DB>;
    static LaunchOnce lds_once;  // per instantiation
    if (rtoss_status st = ensure_dynamic_lds((const void*)kern, smem, lds_once, "conv3x3 shared memory attribute")) return st;
    const int64_t total = (int64_t)tiles_r * tiles_c * co_blocks * c.N;
    if (total > 0x3fffffff) return fail(RTOSS_ESHAPE, "conv: too many tiles");
    if ((int64_t)c.N * c.H * c.W * d.Ci / 8 > 0x7fffffff) return fail(RTOSS_ESHAPE, "conv: input too large for 32-bit chunk offsets");
    const int work_per_xcd = (int)((total + 7) / 8);
    dim3 grid((unsigned)(work_per_xcd * 8)), block(256);
    kern<<<grid, block, smem, s>>>((const T*)x, (TO*)y, wfrag, wfrag + fragment_bytes(d, LAY), c.H, c.W, d.Ci, d.Co, Ho, Wo,
                                   m_tiles_total, tiles_c, tiles_r * tiles_c, co_blocks, (int)total, work_per_xcd, c.ep);
    return check_hip(hipGetLastError(), "conv3x3 sparse launch");
}

// Large stride-1 layers (more than 64 channels in and out, enough 16x16 x 128-channel tiles to give most
// compute units one) take the pipelined kernel of conv3x3_rows.hip.
inline bool takes_pipelined_kernel(const rtoss_wdesc& d, const ConvParams& c)
{
    if (c.stride != 1 || d.Co <= 64 || d.Ci <= 64) return false;
    const int64_t tiles8 = (int64_t)((c.H + 15) / 16) * ((c.W + 15) / 16) * c.N * (((d.Co + 15) / 16 + 7) / 8);
    return tiles8 >= 200;
}

// Layout 1 (three tap groups, 4-entry dictionaries): the single-buffered kernel for every shape.
template <typename T, typename TO>
rtoss_status launch_typed_layout1(const rtoss_wdesc& d, const ConvParams& c, const char* wfrag, const void* x, void* y,
                                  hipStream_t s)
{
    if (c.stride == 1) return launch_variant_sb<T, TO, 1, 4, 2, 2, 4, false, 1>(d, c, wfrag, x, y, s);
    if (d.Ci == 32) return launch_variant_sb<T, TO, 2, 4, 1, 1, 4, false, 1>(d, c, wfrag, x, y, s);
    return launch_variant_sb<T, TO, 2, 4, 2, 2, 4, false, 1>(d, c, wfrag, x, y, s);
}

template <typename T, typename TO>
rtoss_status launch_typed(const rtoss_wdesc& d, const ConvParams& c, const char* wfrag, const void* x, void* y,
                          hipStream_t s)
{
    // The fragment section is padded to a multiple of 8 channel tiles, so any TM <= 8 may over-read rows
    // that hold zeros; outputs beyond Co are never stored.
    // Layers with at most 64 output channels, or too few stages to amortise the pipelined kernel's
    // prologue, come here: 64 channels per workgroup.
    if (c.stride == 1) {
        // 8x16-position tiles for these: 38 KB of LDS per buffer.  (Measured: several resident workgroups beat one
        // workgroup per compute unit with larger buffers, and beat 16x16 tiles, on every such layer.)
        // (up to 64 input channels are one or two stages: nothing to gain inside a workgroup, see AHEAD; one buffer,
        // four workgroups per compute unit)
        if (d.Ci <= 64) return launch_variant_sb<T, TO, 1, 4, 2, 2, 4, false>(d, c, wfrag, x, y, s);
        // deeper layers: two buffers per workgroup (still two workgroups per compute unit); also the launches that
        // would leave compute units idle with the pipelined kernel's 128 channels per workgroup
        return launch_variant_sb<T, TO, 1, 4, 2, 2, 4, true, 0, true>(d, c, wfrag, x, y, s);
    }
    // Stride 2: an output position needs four input positions, so the activation tile dominates the LDS and the
    // copies.  Small tiles of 64 output positions (50 KB with 64 channels per workgroup: three workgroups per compute
    // unit, which overlap each other's copies) measured faster than 8x16 tiles on every stride-2 layer of a
    // YOLOv5s-shaped model; 8x8 where that shape pads the image less than 4x16 (40x40 and 20x20 outputs), else 4x16.
    const int Ho = (c.H - 1) / 2 + 1, Wo = (c.W - 1) / 2 + 1;
    const int64_t padded_4x16 = (int64_t)((Ho + 3) / 4 * 4) * ((Wo + 15) / 16 * 16);
    const int64_t padded_8x8 = (int64_t)((Ho + 7) / 8 * 8) * ((Wo + 7) / 8 * 8);
    if (padded_8x8 < padded_4x16) return launch_variant_sb<T, TO, 2, 4, 1, 2, 2>(d, c, wfrag, x, y, s);
    return launch_variant_sb<T, TO, 2, 4, 1, 1, 4>(d, c, wfrag, x, y, s);
}

}  // namespace

// ---- host-visible entry points of this file ----

int sparse3x3_layout(const Dict& dict)
{
    for (int l = 0; l < kNumLayouts; ++l) {
        bool fits = true;
        for (int g = 0; g < kLayouts[l].groups && fits; ++g) {
            unsigned set = 0;
            for (int f = 0; f < 4; ++f)
                if (kLayouts[l].tap[g][f] >= 0) set |= 1u << kLayouts[l].tap[g][f];
            for (int p = 0; p < dict.P && fits; ++p) fits = __builtin_popcount(dict.mask[p] & set) <= 2;
        }
        if (fits) return l;
    }
    return -1;
}

bool sparse3x3_shape_ok(const rtoss_wdesc& d)
{
    return d.ksize == 3 && (d.dt == RTOSS_F16 || d.dt == RTOSS_BF16) && d.Ci % 32 == 0 && d.Co % 16 == 0;
}

size_t sparse3x3_section_bytes(const rtoss_wdesc& d, int layout)
{
    return fragment_bytes(d, layout) + zero_block_bytes(d);
}

static SparsePackArgs sparse_pack_args(const rtoss_wdesc& d, int layout, const void* w, const uint8_t* idx, void* section,
                                       void* live_values, uint8_t* live_idx, int* blocks)
{
    const int items_per_tile = 64 * layout_fragments(kLayouts[layout]);
    SparsePackArgs a;
    a.w = w;
    a.idx = idx;
    a.out = (char*)section;
    a.Co = d.Co;
    a.Ci = d.Ci;
    a.m_tiles = padded_m_tiles(d.Co);
    a.total_items = (int64_t)(d.Ci / 32) * a.m_tiles * items_per_tile;
    a.zero_items = (int)(zero_block_bytes(d) / 16);
    a.job = make_live_job(live_values, live_idx, (int64_t)d.Co * d.Ci);
    *blocks = (int)(a.job.blocks + a.total_items / items_per_tile + (a.zero_items + 255) / 256);  // public section, tiles, zeros
    return a;
}

rtoss_status launch_pack_sparse3x3(const rtoss_wdesc& d, const void* w, const uint8_t* idx, const Dict& dict,
                                   void* section, void* live_values, uint8_t* live_idx, hipStream_t s)
{
    int blocks = 0;
    const int layout = sparse3x3_layout(dict);
    if (layout < 0) return fail(RTOSS_EINVAL, "pack: the dictionary has no 2-of-4 tap layout");
    const SparsePackArgs a = sparse_pack_args(d, layout, w, idx, section, live_values, live_idx, &blocks);
    dim3 grid((unsigned)blocks), block(256);
    if (d.dt == RTOSS_F16) pack_sparse3x3_kernel<f16_t><<<grid, block, 0, s>>>(a, kLayouts[layout], dict);
    else pack_sparse3x3_kernel<bf16_t><<<grid, block, 0, s>>>(a, kLayouts[layout], dict);
    return check_hip(hipGetLastError(), "pack sparse3x3 launch");
}

rtoss_status launch_pack_sparse3x3_batch(const PackItem* items, int n, const Dict& dict, hipStream_t s)
{
    const int layout = sparse3x3_layout(dict);
    if (layout < 0) return fail(RTOSS_EINVAL, "pack: the dictionary has no 2-of-4 tap layout");
    for (int base = 0; base < n; base += kPackBatchMax) {
        SparsePackBatch b;
        b.layout = kLayouts[layout];
        b.n = std::min(kPackBatchMax, n - base);
        int total = 0;
        for (int i = 0; i < b.n; ++i) {
            const PackItem& it = items[base + i];
            int blocks = 0;
            b.a[i] = sparse_pack_args(it.d, layout, it.w, it.idx, it.section, it.live, it.live_idx, &blocks);
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

rtoss_status launch_conv3x3_sparse(const rtoss_wdesc& d, const ConvParams& c, int layout, const void* section, const void* x,
                                   void* y, hipStream_t s)
{
    const char* wf = (const char*)section;
    const bool f32out = c.out_dt == RTOSS_F32;
    if (layout == 1) {
        if (d.dt == RTOSS_F16)
            return f32out ? launch_typed_layout1<f16_t, float>(d, c, wf, x, y, s) : launch_typed_layout1<f16_t, f16_t>(d, c, wf, x, y, s);
        return f32out ? launch_typed_layout1<bf16_t, float>(d, c, wf, x, y, s) : launch_typed_layout1<bf16_t, bf16_t>(d, c, wf, x, y, s);
    }
    if (layout != 0) return fail(RTOSS_EINVAL, "conv: unknown tap layout %d", layout);
    if (takes_pipelined_kernel(d, c)) return launch_conv3x3_rows(d, c, section, x, y, s);
    if (d.dt == RTOSS_F16)
        return f32out ? launch_typed<f16_t, float>(d, c, wf, x, y, s) : launch_typed<f16_t, f16_t>(d, c, wf, x, y, s);
    return f32out ? launch_typed<bf16_t, float>(d, c, wf, x, y, s) : launch_typed<bf16_t, bf16_t>(d, c, wf, x, y, s);
}

}  // namespace rtoss
