// 3x3 convolution for layers whose kernels share their patterns in blocks (Section IV.A / IV.C: the layers of
// a group take over the kernel patterns of the group's parent, so that kernels with the same pattern can be
// processed together): live taps gathered onto the DENSE matrix instruction.
//
// A dense step D += A * B shares its 32 K-slots between the 16 output channels of A.  Lane quarter q of the B
// operand supplies K = 8q .. 8q+7 with one 16-byte LDS read, i.e. 8 consecutive input channels at ONE tap.  So a
// K-slot can be skipped when a whole block of kernels -- here 64 output channels x 8 input channels -- has the tap
// pruned.  The packer looks at every such block, forms the union U of the live taps of its 512 kernels, and
// emits one dense step per element of U (kernels of the block that lack a tap of U carry an explicit zero
// there).  A stage of 32 input channels is four such blocks side by side, one per lane quarter, each walking
// its own tap list; the stage takes max |U| steps instead of 9.
//   - patterns shared by the block (|U| = k): k steps, every multiply-add a non-zero one -- ceiling 100 % of the
//     dense rate on non-zero work, against k/5 of the 2-of-4 layout and k/9 of dense mode;
//   - independent patterns per kernel (|U| = 9 almost surely): 9 steps, the same work as dense mode.  The result is
//     exact either way; the number of steps is the packer's detection result, stored per (stage, channel block)
//     in the section's header, where the caller can read it.
//
// Section layout: [headers: one GatherHeader per (stage, channel block)][fragments: per (stage, channel block) 9 steps x
// 4 channel fragments x 64 lanes x 16 B, the first `steps` of them written][block of zeros for padding copies].
// Kernel: the dense-mode kernel's data flow (conv3x3_dense.hip: 64 channels x 16x16 positions per workgroup,
// single LDS buffer), with a per-stage step count and a per-quarter tap offset per step.
#include <algorithm>
#include <type_traits>

#include "common.h"
#include "dtypes.h"
#include "epilogue.h"
#include "mma.h"
#include "pack_live.h"
#include "rows_plan.h"
#include "sparse_frag.h"
#include "tile3x3.h"

namespace rtoss {

namespace {

constexpr int kFrag = 1024;  // 64 lanes x 16 bytes = 16 output channels x 32 K-slots of one step
constexpr int kTM = 4;       // channel fragments per channel block (64 output channels)
constexpr int kStepBytes = kTM * kFrag;
constexpr int kBlockBytes = 9 * kStepBytes;
constexpr int kMaxStages = 64;  // headers of one channel block are staged in LDS: Ci <= 2048

struct GatherHeader {     // 64 bytes
    uint32_t steps;       // dense steps of this (stage, channel block): max over the quarters of |U|
    uint8_t count[4];     // |U| of each quarter (8 input channels)
    uint8_t tap[4][9];    // taps of U in ascending order, then repeats of a valid tap (weights there are zero)
    uint8_t pad[20];
};
static_assert(sizeof(GatherHeader) == 64, "header layout is part of the blob format");

inline int channel_blocks(int Co) { return (Co + 16 * kTM - 1) / (16 * kTM); }
inline size_t header_bytes(const rtoss_wdesc& d) { return align_up((size_t)(d.Ci / 32) * channel_blocks(d.Co) * sizeof(GatherHeader), 256); }
inline size_t frag_bytes(const rtoss_wdesc& d) { return (size_t)(d.Ci / 32) * channel_blocks(d.Co) * kBlockBytes; }
inline size_t zero_bytes(const rtoss_wdesc& d) { return align_up((size_t)2 * d.Ci + 16, 256); }

// One workgroup per (stage, channel block) behind the blocks that write the public section.
template <typename T>
__global__ __launch_bounds__(256) void pack_gather3x3_kernel(const T* __restrict__ w, const uint8_t* __restrict__ idx, Dict dict,
                                                             char* __restrict__ section, int Co, int Ci, int cblocks,
                                                             int n_blocks, size_t hdr_bytes, size_t frag_total,
                                                             int zero_items, LiveJob job)
{
    __shared__ uint16_t masks[256];
    __shared__ unsigned uni[4];
    __shared__ GatherHeader hdr;
    masks[threadIdx.x] = dict.mask[threadIdx.x];
    if (threadIdx.x < 4) uni[threadIdx.x] = 0;
    __syncthreads();
    if ((int)blockIdx.x < job.blocks) {  // the first blocks write the blob's public section
        pack_live_block<T>(w, idx, masks, dict.k, job, blockIdx.x);
        return;
    }
    const int b = (int)blockIdx.x - job.blocks;
    if (b >= n_blocks) {  // the blocks behind the fragments write the block of zeros, 16 bytes per lane
        const int item = (b - n_blocks) * 256 + (int)threadIdx.x;
        if (item < zero_items) *(u32x4*)(section + hdr_bytes + frag_total + (size_t)item * 16) = u32x4{0, 0, 0, 0};
        return;
    }
    const int cb = b % cblocks, stage = b / cblocks;
    // ---- union of the live taps of each quarter's 64 x 8 kernels ----
    for (int e = threadIdx.x; e < 64 * 32; e += 256) {
        const int col = e / 32, c = e % 32;  // output channel within the block, input channel within the stage
        const int co = cb * 64 + col;
        if (co < Co) atomicOr(&uni[c / 8], (unsigned)masks[idx[(int64_t)co * Ci + 32 * stage + c]]);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned steps = 0;
        for (int q = 0; q < 4; ++q) {
            int n = 0;
            for (int t = 0; t < 9; ++t)
                if ((uni[q] >> t) & 1u) hdr.tap[q][n++] = (uint8_t)t;
            hdr.count[q] = (uint8_t)n;
            for (int s = n; s < 9; ++s) hdr.tap[q][s] = n ? hdr.tap[q][0] : (uint8_t)4;
            steps = n > (int)steps ? (unsigned)n : steps;
        }
        hdr.steps = steps;
        for (int i = 0; i < 20; ++i) hdr.pad[i] = 0;
    }
    __syncthreads();
    if (threadIdx.x < 16) ((uint32_t*)(section + (size_t)b * sizeof(GatherHeader)))[threadIdx.x] = ((const uint32_t*)&hdr)[threadIdx.x];
    // ---- fragments: [step][fragment m][lane]; row 4q'+i of fragment m is channel 16q' + 4m + i of the block, so that a
    // lane's 16 accumulator values are 16 consecutive channels (as in the dense-mode kernel) ----
    char* out = section + hdr_bytes + (size_t)b * kBlockBytes;
    // (step 0 is always written, zeros when the block has no live tap at all: the pipelined kernel starts every
    // accumulator with it)
    const int items = (int)(hdr.steps ? hdr.steps : 1u) * kTM * 64;
    for (int item = threadIdx.x; item < items; item += 256) {
        const int lane = item % 64, m = (item / 64) % kTM, s = item / (64 * kTM);
        const int r = lane % 16, q = lane / 16;
        const int co = cb * 64 + (r / 4) * 16 + 4 * m + (r % 4);
        const int t = hdr.tap[q][s];
        const bool in_list = s < hdr.count[q];
        T v[8];
        for (int j = 0; j < 8; ++j) {
            __builtin_memset(&v[j], 0, sizeof(T));
            if (co < Co && in_list) {
                const int64_t g = (int64_t)co * Ci + 32 * stage + 8 * q + j;
                if ((masks[idx[g]] >> t) & 1u) v[j] = w[g * 9 + t];
            }
        }
        u32x4 pk;
        __builtin_memcpy(&pk, v, 16);
        *(u32x4*)(out + (size_t)item * 16) = pk;
    }
}

template <typename T, typename TO, int S>
__global__ __launch_bounds__(256) void conv3x3_gather_kernel(const T* __restrict__ x, TO* __restrict__ y,
                                                             const GatherHeader* __restrict__ headers,
                                                             const char* __restrict__ wfrag, const char* __restrict__ zeros,
                                                             int H, int W, int Ci, int Co, int Ho, int Wo, int cblocks,
                                                             int tiles_c, Epilogue ep)
{
    constexpr int RT = 4, CT = 4, TM = kTM;
    using G = Geom<S, RT, CT>;
    constexpr int kTN = RT * CT / 4;  // position blocks per wave
    constexpr int A_COPIES = 9 * TM;  // at most: copy instructions (64 lanes x 16 B) of a stage's fragments
    constexpr int A_PER_WAVE = (A_COPIES + 3) / 4;
    constexpr int X_CHUNKS = G::x_bytes / 16;  // including the pad chunk of every position
    constexpr int X_PER_WAVE = ((X_CHUNKS + 63) / 64 + 3) / 4;
    extern __shared__ __attribute__((aligned(16))) char smem[];  // [weights][activations, rounded up to whole copies][tap offsets]
    char* lds_a = smem;
    char* lds_x = smem + A_PER_WAVE * 4096;
    // per stage: step count, and the LDS offset of every (quarter, step)'s tap
    int* lds_steps = (int*)(lds_x + X_PER_WAVE * 4096);
    int16_t* lds_off = (int16_t*)(lds_steps + kMaxStages);  // [stage][quarter][12]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tile_r = blockIdx.x / tiles_c, tile_c = blockIdx.x % tiles_c;
    const int cb = blockIdx.y, n_img = blockIdx.z;
    const int oh0 = tile_r * G::TH, ow0 = tile_c * G::TW;
    const int ih0 = oh0 * S - 1, iw0 = ow0 * S - 1;
    const int stages = Ci / 32;

    // ---- this channel block's headers -> LDS ----
    for (int e = tid; e < stages * 40; e += 256) {
        const int stage = e / 40, i = e % 40;
        const GatherHeader* h = headers + (size_t)stage * cblocks + cb;
        if (i < 36) {
            const int t = h->tap[i / 9][i % 9];
            lds_off[(stage * 4 + i / 9) * 12 + i % 9] = (int16_t)(((t / 3) * G::LW + (t % 3)) * G::kPos);
        } else if (i == 36) {
            lds_steps[stage] = (int)(h->steps > 9u ? 9u : h->steps);  // (a corrupt header cannot run the loops out of bounds)
        }
    }

    // Copy sources of stage 0.  Every lane copies 16 bytes in every copy instruction; a lane whose LDS
    // slot is zero padding of the tile (or a pad chunk) reads the block of zeros behind the fragments.
    const char* x_ptr[X_PER_WAVE];
#pragma unroll
    for (int k = 0; k < X_PER_WAVE; ++k) {
        const int c = (k * 4 + wave) * 64 + lane;
        const int pos = c / G::kChunks, q = c % G::kChunks;
        const int pr = pos / G::LW, pc = pos % G::LW;
        const int ih = ih0 + pr, iw = iw0 + pc;
        const bool inside = q < 4 && pr < G::IH && pc < G::IW && ih >= 0 && ih < H && iw >= 0 && iw < W;
        x_ptr[k] = inside ? (const char*)x + ((((int64_t)n_img * H + ih) * W + iw) * Ci + q * 8) * 2 : zeros;
    }
    const char* a_src = wfrag + (int64_t)cb * kBlockBytes + lane * 16;
    const int64_t a_stage_stride = (int64_t)cblocks * kBlockBytes;

    const int nn = lane & 15, qq = lane >> 4;
    const int pr = nn >> 2, pc = nn & 3;
    int xb[kTN];  // LDS byte offset of this lane's position in each of its blocks, tap (0,0), its 8 channels
#pragma unroll
    for (int j = 0; j < kTN; ++j) {
        const int blk = wave * kTN + j;
        xb[j] = (((4 * (blk / CT) + pr) * S) * G::LW + (4 * (blk % CT) + pc) * S) * G::kPos + qq * 16;
    }

    f32x4 acc[TM][kTN];
#pragma unroll
    for (int m = 0; m < TM; ++m)
#pragma unroll
        for (int j = 0; j < kTN; ++j) acc[m][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    for (int stage = 0; stage < stages; ++stage) {
        __syncthreads();  // everybody is done reading the previous stage (and, the first time, the headers are in LDS)
        const int steps = lds_steps[stage];  // uniform
        const int a_copies = steps * TM;
#pragma unroll
        for (int k = 0; k < A_PER_WAVE; ++k) {
            const int kk = k * 4 + wave;
            if (kk < a_copies) copy16_to_lds(a_src + stage * a_stage_stride + kk * 1024, lds_a + kk * 1024);  // wave-uniform
        }
#pragma unroll
        for (int k = 0; k < X_PER_WAVE; ++k) copy16_to_lds(x_ptr[k] + stage * 64, lds_x + (k * 4 + wave) * 1024);
        __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): this wave's copies have landed in LDS
        __syncthreads();                     // ... and everybody's
        const int16_t* my_off = lds_off + (stage * 4 + qq) * 12;
        for (int s = 0; s < steps; ++s) {
            const int off = my_off[s];  // this quarter's tap of step s
            u32x4 b[kTN];
#pragma unroll
            for (int j = 0; j < kTN; ++j) b[j] = *(const u32x4*)(lds_x + xb[j] + off);
#pragma unroll
            for (int m = 0; m < TM; ++m) {
                const u32x4 a = *(const u32x4*)(lds_a + (s * TM + m) * kFrag + lane * 16);
#pragma unroll
                for (int j = 0; j < kTN; ++j) acc[m][j] = Dense16<T>::mma(a, b[j], acc[m][j]);
            }
        }
    }

    // ---- store: 16 consecutive channels of this lane's position in each of its blocks ----
    const int co_lane = cb * (16 * kTM) + 16 * qq;
    constexpr int EB = (int)sizeof(TO);
    constexpr int RUN = 4 * TM;
#pragma unroll
    for (int j = 0; j < kTN; ++j) {
        const int blk = wave * kTN + j;
        const int oh = oh0 + 4 * (blk / CT) + pr, ow = ow0 + 4 * (blk % CT) + pc;
        if (oh >= Ho || ow >= Wo || co_lane >= Co) continue;  // Co is a multiple of 16: a run is all in or all out
        const int64_t pos = ((int64_t)n_img * Ho + oh) * Wo + ow;
        TO* yp = y + pos * ep.ldy + co_lane;
        float v[RUN];
#pragma unroll
        for (int m = 0; m < TM; ++m)
#pragma unroll
            for (int e = 0; e < 4; ++e) v[4 * m + e] = acc[m][j][e];
        epi_scale_bias_act<RUN>(v, ep, co_lane);
        epi_residual<TO, RUN>(v, ep, pos, co_lane);
        if constexpr (EB == 4) {
#pragma unroll
            for (int g = 0; g < TM; ++g) *(f32x4*)(yp + 4 * g) = f32x4{v[4 * g], v[4 * g + 1], v[4 * g + 2], v[4 * g + 3]};
        } else {
#pragma unroll
            for (int g = 0; g < TM / 2; ++g) {
                u32x4 o;
                o.x = pack2_from_f32<TO>(v[8 * g + 0], v[8 * g + 1]);
                o.y = pack2_from_f32<TO>(v[8 * g + 2], v[8 * g + 3]);
                o.z = pack2_from_f32<TO>(v[8 * g + 4], v[8 * g + 5]);
                o.w = pack2_from_f32<TO>(v[8 * g + 6], v[8 * g + 7]);
                *(u32x4*)(yp + 8 * g) = o;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------------------
// Pipelined variant over strips of rows: the tiling, persistent workgroups, double-buffered stages and direct
// epilogue of conv3x3_rows.hip (stride 1, 128 output channels x 16 columns x 4*TN rows per workgroup), around a
// much simpler stage.  The workgroup is 8 waves, two per SIMD: wave (v, h) owns TN rows of the tile and block h of
// the pair of 64-channel blocks, with that block's own tap lists.  A step is 4*TN dense matrix instructions on
// operands read straight from LDS at the start of the step -- four weight fragments and one 16-byte activation
// read per output row (the step's tap is a per-quarter LDS offset), no transposes, no prefetch registers: the
// partner wave's matrix instructions cover the reads.  (Eight waves leave each 128 vector registers next to its
// 80 accumulators; a four-wave form with the operands of the next half-step prefetched into a second register
// set measured 5 % slower.)  Up to kGrSteps steps of a stage live in LDS; a tile with more, or with different
// counts in its blocks or stages (patterns that are not shared after all), takes the general body: weight
// fragments from global memory, slowly but correctly.
// ---------------------------------------------------------------------------------------------------------
constexpr int kGrSteps = 5;
constexpr int kGrWaves = 8;                           // two per SIMD: wave = (row group, block of the pair)
constexpr int kGrABytes = kGrSteps * 2 * kStepBytes;  // [step][block of the pair][fragment]: 40 KB
constexpr int kGrXChunks = (4 * kTall + 2) * kLW * 4;
constexpr int kGrXPerWave = ((kGrXChunks + 63) / 64 + kGrWaves - 1) / kGrWaves;
constexpr int kGrXArea = kGrXPerWave * kGrWaves * 1024;
constexpr int kGrRegion = kGrABytes + kGrXArea;
constexpr int kGrAPerWave = kGrABytes / 1024 / kGrWaves;
constexpr int kGrCopySlots = kGrAPerWave + kGrXPerWave;
constexpr int kGrOffPitch = 8;  // int16 entries per (stage, block, quarter): steps 0..7, one 16-byte read
constexpr size_t kGrSmem = 2 * (size_t)kGrRegion + kMaxStages * 4 + (size_t)kMaxStages * 2 * 4 * kGrOffPitch * 2;
static_assert(kGrABytes / 1024 == kGrAPerWave * kGrWaves, "every wave issues the same number of weight copies");
static_assert(kMaxStages * 8 <= 64 * kGrWaves, "one table entry per thread");

__device__ __forceinline__ int pair_block(int cb0, int half, int cblocks) { return cb0 + (half && cb0 + 1 < cblocks ? 1 : 0); }

template <typename T, typename TO>
__global__ __launch_bounds__(64 * kGrWaves, 1) void conv3x3_gather_rows_kernel(const T* __restrict__ x, TO* __restrict__ y,
                                                                                const GatherHeader* __restrict__ headers,
                                                                                const char* __restrict__ wfrag,
                                                                                const char* __restrict__ zeros, int H, int W,
                                                                                int Ci, int Co, int cblocks, RowPlan plan,
                                                                                float relu_floor, int ldy)
{
    static_assert(sizeof(TO) == 2, "direct epilogue: 16-bit output");
    extern __shared__ __attribute__((aligned(16))) char smem[];  // two regions, then the tile's step counts and tap offsets
    int* lds_steps = (int*)(smem + 2 * kGrRegion);               // [stage]: steps of block 0 | steps of block 1 << 8
    int16_t* lds_off = (int16_t*)(lds_steps + kMaxStages);       // [stage][block][quarter][kGrOffPitch]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int vrow = wave & 3;   // which TN rows of the tile
    const int hsel = wave >> 2;  // which 64-channel block of the pair
    const int stages = Ci / 32;
    const int Ho = H, Wo = W;  // stride 1, padding 1

    // ---- this workgroup's entries (as in conv3x3_rows.hip) ----
    const int xcd = blockIdx.x % 8, slot = blockIdx.x / 8, slots = gridDim.x / 8;
    const int tall_end = min((xcd + 1) * plan.tall_per_xcd, plan.tall_total);
    const int short_end = min((xcd + 1) * plan.short_per_xcd, plan.short_total);
    int tall_next = xcd * plan.tall_per_xcd + slot;
    int short_next = xcd * plan.short_per_xcd + (slots - 1 - slot);
    if (tall_next >= tall_end && short_next >= short_end) return;

    // ---- copy state: the tile whose stages are being fetched ----
    int c_cb0 = 0;
    const char* x_ptr[kGrXPerWave];
    // A lane's source of activation copy slot k for tile t, in four parts (position in the tile; image coordinates
    // and chunk number; address; zero padding), as in conv3x3_rows.hip: the first tile does them in one go, the last
    // stage of a tile spreads the next tile's over its matrix instructions.  The empty asm statements pin each
    // part's results where it is written (they are ordered with the matrix instructions).
    int sp_a = 0, sp_b = 0, sp_off = 0;
    const char* sp_addr = nullptr;
    auto source_part = [&](auto K, auto P, const TileCoord& t, int in_rows) {
        constexpr int k = decltype(K)::value, part = decltype(P)::value;
        if constexpr (part == 0) {
            int l = lane;
            asm volatile("" : "+v"(l));  // recomputed here rather than kept in registers through the K loop
            const int pos = (k * kGrWaves + wave) * 16 + (l >> 2);
            sp_a = pos / kLW;
            sp_b = pos - sp_a * kLW;
            asm volatile("" : "+v"(sp_a), "+v"(sp_b));
        } else if constexpr (part == 1) {
            sp_a += t.oh0 - 1;  // input row and column
            sp_b += t.ow0 - 1;
            sp_off = ((t.n_img * H + sp_a) * W + sp_b) * (Ci >> 3) + (lane & 3);  // 16-byte chunks: fits 31 bits (launcher)
            asm volatile("" : "+v"(sp_a), "+v"(sp_b), "+v"(sp_off));
        } else if constexpr (part == 2) {
            sp_addr = (const char*)x + (int64_t)sp_off * 16;
            asm volatile("" : "+v"(sp_addr));
        } else {
            const int row_end = min(H, t.oh0 - 1 + in_rows);  // rows of the tile, and of the image
            const bool inside = (unsigned)sp_a < (unsigned)row_end && (unsigned)sp_b < (unsigned)W;
            x_ptr[k] = inside ? sp_addr : zeros;
            asm volatile("" : "+v"(x_ptr[k]));
        }
    };
    constexpr int kSourceParts = 4 * kGrXPerWave;
    auto setup_tile_sources = [&](const TileCoord& t, int in_rows) {
        static_for<kSourceParts>([&](auto PN) {
            constexpr int pn = decltype(PN)::value;
            source_part(std::integral_constant<int, pn / 4>{}, std::integral_constant<int, pn % 4>{}, t, in_rows);
        });
    };
    // One copy instruction (64 lanes x 16 bytes) of stage `stage` of the copy state's tile into region `par`: slots
    // 0 .. kGrAPerWave-1 move weight fragments (a_src: this wave's block's fragments of that stage), the rest activations.
    auto issue_copy_slot = [&](int cslot, int stage, int par, const char* a_src) {
        // (the LDS address of a copy travels in a scalar register: keep the region's offset scalar)
        char* region = smem + __builtin_amdgcn_readfirstlane(par * kGrRegion);
        if (cslot < kGrAPerWave) {
            // piece 8 * cslot + wave of the region is (step, block, fragment) = (cslot, wave / 4, wave % 4).  All
            // kGrSteps steps are copied whatever the stage's own count (what lies behind a block's last step in the
            // blob is never multiplied): a count would put a branch around every copy, and branches between the
            // matrix instructions cost more than the surplus copies.
            copy16_to_lds(a_src + (cslot * kTM + vrow) * kFrag, region + (cslot * kGrWaves + wave) * 1024);
        } else {
            const int k = cslot - kGrAPerWave;
            copy16_to_lds(x_ptr[k] + stage * 64, region + kGrABytes + (k * kGrWaves + wave) * 1024);
        }
    };
    // this wave's share of the weight fragments of stage `stage` of the copy state's tile: fragment wave % 4 of its
    // block (no second block in the pair: the first one again, never stored)
    auto weight_source = [&](int stage) {
        return wfrag + ((int64_t)stage * cblocks + pair_block(c_cb0, hsel, cblocks)) * kBlockBytes + lane * 16;
    };

    const int nn = lane & 15, qq = lane >> 4;
    f32x4 acc[kTM][kTall];
    u32x4 a_op[kTM], b_op[kTall];  // operands of the step being multiplied (the partner wave on the SIMD covers their latency)
    int gpar = 0;                        // region that holds the stage about to be multiplied

    // A tile's table entries (stage, block of the pair, quarter): the offsets in the activation tile of the taps of
    // steps 0..7, and per stage the two step counts.  A thread fetches one entry from the headers in global memory
    // into registers (prefetch_headers, a tile ahead) and writes it to LDS when the tile starts.
    u32x4 hdr_off;
    int hdr_steps;
    auto prefetch_headers = [&](int cb0) {
        hdr_off = u32x4{0, 0, 0, 0};
        hdr_steps = 0;
        if (tid < stages * 8) {
            const int stage = tid >> 3, half = (tid >> 2) & 1, q = tid & 3;
            const GatherHeader* h = headers + (size_t)stage * cblocks + pair_block(cb0, half, cblocks);
            uint32_t o[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int t = h->tap[q][i];
                o[i] = (uint32_t)(((t / 3) * kLW + (t % 3)) * kPosBytes);
            }
            hdr_off = u32x4{o[0] | (o[1] << 16), o[2] | (o[3] << 16), o[4] | (o[5] << 16), o[6] | (o[7] << 16)};
            if (half == 0 && q == 0) {
                const GatherHeader* h0 = headers + (size_t)stage * cblocks + cb0;
                unsigned s0 = h0->steps, s1 = cb0 + 1 < cblocks ? h0[1].steps : 0u;
                s0 = s0 > 9u ? 9u : s0;  // (a corrupt header cannot run the loops out of bounds)
                s1 = s1 > 9u ? 9u : s1;
                if (stage == 0) {  // every accumulator starts with step 0
                    s0 = s0 ? s0 : 1u;
                    s1 = s1 ? s1 : 1u;
                }
                hdr_steps = (int)(s0 | (s1 << 8));
            }
        }
    };
    auto store_headers = [&]() {
        if (tid < stages * 8) {
            *(u32x4*)(lds_off + tid * kGrOffPitch) = hdr_off;
            if ((tid & 7) == 0) lds_steps[tid >> 3] = hdr_steps;
        }
    };

    // ---- one tile of TN rows per wave ----
    auto run_tile = [&](auto tn_tag, const TileCoord& cur, bool has_next, const TileCoord& nxt, bool nxt_tall) {
        constexpr int TN = decltype(tn_tag)::value;
        const int xrd = ((vrow * TN) * kLW + nn) * kPosBytes + qq * 16;
        const int nxt_in_rows = nxt_tall ? 4 * kTall + 2 : 4 * kShort + 2;
        const int cb0 = cur.mt0 / kTM;

        // the tile's step counts and tap offsets, fetched from the headers while the previous tile was still being
        // multiplied, -> LDS (nobody reads the previous tile's any more: its last stage ended at a barrier)
        store_headers();
        __syncthreads();

        // A stage's tap offsets (steps 0..7 of this wave's block, this lane's quarter) are read one stage ahead into
        // registers, so that no operand read waits for a table look-up.
        auto load_offsets = [&](int stage) -> u32x4 {
            return *(const u32x4*)(lds_off + ((stage * 2 + hsel) * 4 + qq) * kGrOffPitch);
        };
        auto offset_of = [](const u32x4& pk, int st) -> int {  // st < 8, compile-time after unrolling
            return (int)((pk[st >> 1] >> ((st & 1) * 16)) & 0xffffu);
        };
        // operands of a step: the block's four weight fragments and, per output row, this quarter's tap
        auto load_operands = [&](int par, int st, int off, u32x4 (&a)[kTM], u32x4 (&b)[kTall]) {
            const int region = __builtin_amdgcn_readfirstlane(par * kGrRegion);
            const char* A = smem + region + lane * 16 + ((st * 2) * kTM) * kFrag + hsel * (kTM * kFrag);
            const char* X = smem + region + kGrABytes + xrd + off;
#pragma unroll
            for (int m = 0; m < kTM; ++m) a[m] = *(const u32x4*)(A + m * kFrag);
#pragma unroll
            for (int j = 0; j < TN; ++j) b[j] = *(const u32x4*)(X + j * kLW * kPosBytes);
        };
        u32x4 off_cur = load_offsets(0), off_nxt = off_cur;

        auto run_stage = [&](auto first_tag, auto last_tag, auto body_tag, int stage) {
            constexpr bool FIRST = decltype(first_tag)::value, LAST = decltype(last_tag)::value;
            constexpr int BODY = decltype(body_tag)::value;  // steps of the branch-free body, 0: the general body
            // bodies of two steps or more work the next tile's activation sources out between their matrix instructions
            constexpr bool SPREAD_SOURCES = LAST && BODY > 1;
            const int st = __builtin_amdgcn_readfirstlane(lds_steps[stage]);
            const int my_steps = hsel ? st >> 8 : st & 0xff, steps = max(st & 0xff, st >> 8);
            const int copy_stage = LAST ? 0 : stage + 1;
            // (in the very last stage of the last tile nothing is left to fetch; `nxt` is the same tile then and its
            // stage 0 is fetched again into the free region, which keeps this code free of branches)
            if constexpr (LAST) {
                c_cb0 = nxt.mt0 / kTM;
                prefetch_headers(nxt.mt0 / kTM);
                if constexpr (!SPREAD_SOURCES) setup_tile_sources(nxt, nxt_in_rows);
            } else {
                off_nxt = load_offsets(stage + 1);
            }
            const char* const a_src = weight_source(copy_stage);
            auto multiply = [&](auto first_step_tag, const u32x4 (&a)[kTM], const u32x4 (&b)[kTall], auto&& between) {
                static_for<kTM * TN>([&](auto I) {
                    constexpr int i = decltype(I)::value, m = i / TN, j = i % TN;
                    if constexpr (decltype(first_step_tag)::value) Mat<T>::dense_first(a[m], b[j], acc[m][j]);
                    else Mat<T>::dense(a[m], b[j], acc[m][j]);
                    between(I);
                    __builtin_amdgcn_sched_barrier(0);
                });
            };
            // Stage hand-over: every copy of the next stage issued, this wave's landed and its reads of this region
            // done, a bare barrier.
            auto hand_over = [&](int first_unissued) {
                static_for<kGrCopySlots>([&](auto C) {
                    constexpr int c = decltype(C)::value;
                    if (c >= first_unissued) issue_copy_slot(c, copy_stage, gpar ^ 1, a_src);
                });
                asm volatile("" ::: "memory");
                __builtin_amdgcn_s_waitcnt(0x0070);  // vmcnt(0) lgkmcnt(0)
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
            };
            // A tile whose stages all take the same number of steps, at most kGrSteps, in both blocks -- every tile,
            // when the patterns are shared the way the packer hopes -- runs a body without a single branch: STEPS is
            // a compile-time constant, the copies of the next stage are dealt over the early steps and the hand-over
            // sits between the last step's operand reads and its matrix instructions.  (With branches between the
            // steps the compiler's wait-count bookkeeping falls back to waiting for every outstanding LDS read in
            // front of each block of matrix instructions.)  Operands are read at the start of the step that uses them:
            // two waves share a SIMD, and one's matrix instructions cover the other's reads.
            auto static_body = [&](auto steps_tag) {
                constexpr int STEPS = decltype(steps_tag)::value;
                constexpr int CS = STEPS > 2 ? STEPS / 2 : 1;  // steps that carry copies (the early ones)
                static_for<STEPS>([&](auto S) {
                    constexpr int s = decltype(S)::value;
                    constexpr int c0 = (s < CS ? s : CS) * kGrCopySlots / CS, c1 = (s + 1 < CS ? s + 1 : CS) * kGrCopySlots / CS;
                    constexpr int n = STEPS > 1 ? c1 - c0 : 0, total = kTM * TN;
                    load_operands(gpar, s, offset_of(off_cur, s), a_op, b_op);
                    if constexpr (s + 1 == STEPS) hand_over(STEPS > 1 ? kGrCopySlots : 0);
                    multiply(std::integral_constant<bool, FIRST && s == 0>{}, a_op, b_op, [&](auto I) {
                        constexpr int i = decltype(I)::value;
                        if constexpr (SPREAD_SOURCES && s == 0) {
                            // part pn behind matrix instruction pn * D / parts of step 0, in order (the parts share
                            // their temporaries); D: the instruction behind which the last activation copy is issued
                            // when step 0 carries all copies (slot c of n goes behind instruction c * total / n)
                            constexpr int D = CS == 1 ? (kGrCopySlots - 1) * total / kGrCopySlots : total;
                            static_for<kSourceParts>([&](auto PN) {
                                constexpr int pn = decltype(PN)::value;
                                if constexpr (i == pn * D / kSourceParts)
                                    source_part(std::integral_constant<int, pn / 4>{}, std::integral_constant<int, pn % 4>{}, nxt, nxt_in_rows);
                            });
                        }
                        if constexpr (s + 1 < STEPS) {
                            static_for<(n > 0 ? n : 0)>([&](auto K) {
                                constexpr int k = decltype(K)::value;
                                if constexpr (i == k * total / (n > 0 ? n : 1)) issue_copy_slot(c0 + k, copy_stage, gpar ^ 1, a_src);
                            });
                        }
                    });
                });
            };
            // The general body, for tiles whose patterns are not shared the way the packer hopes (any step counts, up
            // to 9, different between the blocks): plain and slow.  Every copy of the next stage first; then a loop
            // over the steps with the weight fragments read from global memory (so that it does not matter how many
            // of them the region holds) and the matrix instructions unconditional: a block that has no step s
            // multiplies by zero, which keeps the accumulators out of every branch.
            auto generic_body = [&]() {
                static_for<kGrCopySlots>([&](auto C) { issue_copy_slot(decltype(C)::value, copy_stage, gpar ^ 1, a_src); });
                const char* X = smem + __builtin_amdgcn_readfirstlane(gpar * kGrRegion) + kGrABytes + xrd;
                const int cb = pair_block(cb0, hsel, cblocks);
                auto step = [&](auto first_step_tag, int st_i) {
                    const char* Ag = wfrag + ((int64_t)stage * cblocks + cb) * kBlockBytes + (st_i * kTM) * kFrag + lane * 16;
                    u32x4 a[kTM], b[kTall];
#pragma unroll
                    for (int m = 0; m < kTM; ++m) a[m] = u32x4{0, 0, 0, 0};
                    if (st_i < my_steps) {  // uniform; fragments past a block's own steps are not written
#pragma unroll
                        for (int m = 0; m < kTM; ++m) a[m] = *(const u32x4*)(Ag + m * kFrag);
                    }
                    int off;
                    if (st_i < 8) {
                        off = lds_off[((stage * 2 + hsel) * 4 + qq) * kGrOffPitch + st_i];
                    } else {  // the table holds steps 0..7
                        const int t = headers[(size_t)stage * cblocks + cb].tap[qq][8];
                        off = ((t / 3) * kLW + (t % 3)) * kPosBytes;
                    }
#pragma unroll
                    for (int j = 0; j < TN; ++j) b[j] = *(const u32x4*)(X + j * kLW * kPosBytes + off);
                    multiply(first_step_tag, a, b, [](auto) {});
                };
                step(std::integral_constant<bool, FIRST>{}, 0);
                for (int st_i = 1; st_i < steps; ++st_i) step(std::false_type{}, st_i);
                hand_over(kGrCopySlots);
            };
            if constexpr (BODY > 0) static_body(body_tag);
            else generic_body();
            off_cur = off_nxt;
            gpar ^= 1;
        };

        // One path per tile: the stages and the epilogue for a given body.  (Choosing the body per stage would join
        // the paths while the accumulators are live; the compiler then moves accumulators between the registers the
        // paths happen to use, right behind matrix instructions whose latency it does not know.)
        auto tile_path = [&](auto body_tag) {
            run_stage(std::true_type{}, std::false_type{}, body_tag, 0);  // (the launcher admits Ci >= 96: three stages or more)
            for (int stage = 1; stage + 1 < stages; ++stage) run_stage(std::false_type{}, std::false_type{}, body_tag, stage);
            run_stage(std::false_type{}, std::true_type{}, body_tag, stages - 1);

            // the last matrix instructions must have written their accumulators before anything reads them
            asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
            // ---- epilogue: a lane holds 16 consecutive channels of its block for column nn of each of its rows
            // (the packer dealt the rows that way): 32 contiguous bytes per lane ----
            {
                int lane_e = lane;
                asm volatile("" : "+v"(lane_e));
                const int nn_e = lane_e & 15, qq_e = lane_e >> 4;
                const int row_first = cur.oh0 + vrow * TN;
                const int64_t pos_tile = ((int64_t)cur.n_img * Ho + cur.oh0) * Wo + cur.ow0;
                TO* const y_tile = y + pos_tile * ldy;
                const bool col_inside = cur.ow0 + nn_e < Wo;
                const int co_lane = 16 * (cur.mt0 + kTM * hsel) + 16 * qq_e;
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const bool inside = col_inside && row_first + j < Ho;
                    TO* yp = y_tile + ((vrow * TN + j) * Wo + nn_e) * ldy + co_lane;
                    uint32_t o[8];
#pragma unroll
                    for (int m = 0; m < kTM; ++m) {
                        float r[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) asm("v_max_f32 %0, %1, %2" : "=v"(r[e]) : "v"(acc[m][j][e]), "v"(relu_floor));
                        o[2 * m] = pack2_from_f32<TO>(r[0], r[1]);
                        o[2 * m + 1] = pack2_from_f32<TO>(r[2], r[3]);
                    }
                    if (inside && co_lane < Co) {
                        *(u32x4*)(yp) = u32x4{o[0], o[1], o[2], o[3]};
                        *(u32x4*)(yp + 8) = u32x4{o[4], o[5], o[6], o[7]};
                    }
                }
            }
        };
        // every stage with the same number of steps in both blocks (one table entry per lane)?
        const int st_first = __builtin_amdgcn_readfirstlane(lds_steps[0]);
        const int st_mine = lds_steps[lane < stages ? lane : 0];
        const bool uniform_steps = __ballot(st_mine != st_first) == 0 && (st_first & 0xff) == (st_first >> 8);
        switch (uniform_steps ? (st_first & 0xff) : 0) {
        case 1: tile_path(std::integral_constant<int, 1>{}); break;
        case 2: tile_path(std::integral_constant<int, 2>{}); break;
        case 3: tile_path(std::integral_constant<int, 3>{}); break;
        case 4: tile_path(std::integral_constant<int, 4>{}); break;
        case 5: tile_path(std::integral_constant<int, 5>{}); break;
        default: tile_path(std::integral_constant<int, 0>{}); break;
        }
    };

    // ---- walk the entries ----
    bool cur_tall = tall_next < tall_end;
    TileCoord cur = decode_entry(plan, cur_tall, cur_tall ? tall_next : short_next);
    if (cur_tall) tall_next += slots;
    else short_next += slots;
    prefetch_headers(cur.mt0 / kTM);
    c_cb0 = cur.mt0 / kTM;
    setup_tile_sources(cur, cur_tall ? 4 * kTall + 2 : 4 * kShort + 2);
    {
        const char* const a_src = weight_source(0);
#pragma unroll
        for (int c = 0; c < kGrCopySlots; ++c) issue_copy_slot(c, 0, 0, a_src);
    }
    bool first_tile = true;
    for (;;) {
        const bool nxt_tall = tall_next < tall_end;
        const bool has_next = nxt_tall || short_next < short_end;
        TileCoord nxt = cur;
        if (has_next) {
            nxt = decode_entry(plan, nxt_tall, nxt_tall ? tall_next : short_next);
            if (nxt_tall) tall_next += slots;
            else short_next += slots;
        }
        if (first_tile) {
            __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): this wave's copies have landed in LDS
            __syncthreads();                     // ... and everybody's
            first_tile = false;
        }
        if (cur_tall) run_tile(std::integral_constant<int, kTall>{}, cur, has_next, nxt, nxt_tall);
        else run_tile(std::integral_constant<int, kShort>{}, cur, has_next, nxt, nxt_tall);
        if (!has_next) break;
        cur = nxt;
        cur_tall = nxt_tall;
    }
}

template <typename T, typename TO, int S>
rtoss_status launch_gather(const rtoss_wdesc& d, const ConvParams& c, const char* section, const void* x, void* y, hipStream_t s)
{
    using G = Geom<S, 4, 4>;
    const int Ho = (c.H + 2 - 3) / S + 1, Wo = (c.W + 2 - 3) / S + 1;
    const int tiles_r = (Ho + G::TH - 1) / G::TH, tiles_c = (Wo + G::TW - 1) / G::TW;
    const int cblocks = channel_blocks(d.Co);
    constexpr int x_copies_per_wave = ((G::x_bytes / 16 + 63) / 64 + 3) / 4;
    constexpr int a_copies_per_wave = (kTM * 9 + 3) / 4;
    const size_t smem = (size_t)(a_copies_per_wave + x_copies_per_wave) * 4096 + kMaxStages * 4 + kMaxStages * 4 * 12 * 2;
    auto kern = conv3x3_gather_kernel<T, TO, S>;
    static LaunchOnce lds_once;  // per instantiation
    if (rtoss_status st = ensure_dynamic_lds((const void*)kern, smem, lds_once, "conv3x3 gather shared memory attribute")) return st;
    if (c.N > 65535 || cblocks > 65535) return fail(RTOSS_ESHAPE, "conv: batch or channel count too large");
    dim3 grid((unsigned)(tiles_r * tiles_c), (unsigned)cblocks, (unsigned)c.N), block(256);
    const char* frags = section + header_bytes(d);
    kern<<<grid, block, smem, s>>>((const T*)x, (TO*)y, (const GatherHeader*)section, frags, frags + frag_bytes(d), c.H, c.W,
                                   d.Ci, d.Co, Ho, Wo, cblocks, tiles_c, c.ep);
    return check_hip(hipGetLastError(), "conv3x3 gather launch");
}

// Large stride-1 layers with 16-bit output and no fused output stage beyond ReLU take the pipelined kernel (the
// same test of size as for the pipelined 2-of-4 kernel: enough 128-channel tiles to give most compute units one).
inline bool takes_pipelined_gather(const rtoss_wdesc& d, const ConvParams& c)
{
    if (c.stride != 1 || d.Co <= 64 || d.Ci <= 64 || c.out_dt == RTOSS_F32) return false;
    if (c.ep.scale || c.ep.bias || c.ep.residual || c.ep.act > 1) return false;
    const int64_t tiles8 = (int64_t)((c.H + 15) / 16) * ((c.W + 15) / 16) * c.N * (((d.Co + 15) / 16 + 7) / 8);
    return tiles8 >= 200;
}

template <typename T>
rtoss_status launch_gather_rows(const rtoss_wdesc& d, const ConvParams& c, const char* section, const void* x, void* y, hipStream_t s)
{
    auto kern = conv3x3_gather_rows_kernel<T, T>;
    static LaunchOnce lds_once;  // per instantiation
    if (rtoss_status st = ensure_dynamic_lds((const void*)kern, kGrSmem, lds_once, "conv3x3 gather shared memory attribute")) return st;
    DeviceInfo dev;
    if (rtoss_status st = current_device(&dev)) return st;
    const int co_blocks = ((d.Co + 15) / 16 + kRowsTM - 1) / kRowsTM;
    if (c.stride != 1 || d.Ci % 32 || d.Ci < 96) return fail(RTOSS_ESHAPE, "conv: the pipelined kernel needs stride 1 and three or more stages of 32 input channels");
    if ((int64_t)c.N * c.H * c.W * d.Ci / 8 > 0x7fffffff) return fail(RTOSS_ESHAPE, "conv: input too large for 32-bit chunk offsets");
    if ((int64_t)c.N * ((c.W + 15) / 16) * ((c.H + 15) / 16 + 1) * co_blocks > 0x3fffffff) return fail(RTOSS_ESHAPE, "conv: too many tiles");
    int slots = 0;
    const RowPlan plan = plan_rows_for_device(c.N, c.H, c.W, co_blocks, d.Ci / 32, dev.cus, &slots);
    const char* frags = section + header_bytes(d);
    const float relu_floor = c.ep.act == 1 ? 0.f : -__builtin_inff();
    dim3 grid((unsigned)(slots * 8)), block(64 * kGrWaves);
    kern<<<grid, block, kGrSmem, s>>>((const T*)x, (T*)y, (const GatherHeader*)section, frags, frags + frag_bytes(d), c.H, c.W, d.Ci,
                                      d.Co, channel_blocks(d.Co), plan, relu_floor, c.ep.ldy);
    return check_hip(hipGetLastError(), "conv3x3 gather rows launch");
}

template <typename T, typename TO>
rtoss_status launch_typed(const rtoss_wdesc& d, const ConvParams& c, const char* section, const void* x, void* y, hipStream_t s)
{
    if constexpr (std::is_same<T, TO>::value)
        if (takes_pipelined_gather(d, c)) return launch_gather_rows<T>(d, c, section, x, y, s);
    if (c.stride == 1) return launch_gather<T, TO, 1>(d, c, section, x, y, s);
    return launch_gather<T, TO, 2>(d, c, section, x, y, s);
}

}  // namespace

// ---- host-visible entry points of this file ----

bool gather3x3_shape_ok(const rtoss_wdesc& d)
{
    return d.ksize == 3 && (d.dt == RTOSS_F16 || d.dt == RTOSS_BF16) && d.Ci % 32 == 0 && d.Ci / 32 <= kMaxStages && d.Co % 16 == 0;
}

size_t gather3x3_header_bytes(const rtoss_wdesc& d) { return header_bytes(d); }
size_t gather3x3_section_bytes(const rtoss_wdesc& d) { return header_bytes(d) + frag_bytes(d) + zero_bytes(d); }

rtoss_status launch_pack_gather3x3(const rtoss_wdesc& d, const void* w, const uint8_t* idx, const Dict& dict, void* section,
                                   void* live_values, uint8_t* live_idx, hipStream_t s)
{
    const LiveJob job = make_live_job(live_values, live_idx, (int64_t)d.Co * d.Ci);
    const int cblocks = channel_blocks(d.Co);
    const int n_blocks = (d.Ci / 32) * cblocks;
    const int zero_items = (int)(zero_bytes(d) / 16);
    dim3 grid((unsigned)(job.blocks + n_blocks + (zero_items + 255) / 256)), block(256);
    if (d.dt == RTOSS_F16)
        pack_gather3x3_kernel<f16_t><<<grid, block, 0, s>>>((const f16_t*)w, idx, dict, (char*)section, d.Co, d.Ci, cblocks, n_blocks,
                                                            header_bytes(d), frag_bytes(d), zero_items, job);
    else
        pack_gather3x3_kernel<bf16_t><<<grid, block, 0, s>>>((const bf16_t*)w, idx, dict, (char*)section, d.Co, d.Ci, cblocks, n_blocks,
                                                             header_bytes(d), frag_bytes(d), zero_items, job);
    return check_hip(hipGetLastError(), "pack gather3x3 launch");
}

rtoss_status launch_conv3x3_gather(const rtoss_wdesc& d, const ConvParams& c, const void* section, const void* x, void* y,
                                   hipStream_t s)
{
    const char* sec = (const char*)section;
    const bool f32out = c.out_dt == RTOSS_F32;
    if (d.dt == RTOSS_F16)
        return f32out ? launch_typed<f16_t, float>(d, c, sec, x, y, s) : launch_typed<f16_t, f16_t>(d, c, sec, x, y, s);
    return f32out ? launch_typed<bf16_t, float>(d, c, sec, x, y, s) : launch_typed<bf16_t, bf16_t>(d, c, sec, x, y, s);
}

}  // namespace rtoss
