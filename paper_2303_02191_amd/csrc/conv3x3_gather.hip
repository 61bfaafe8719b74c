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
    const int items = (int)hdr.steps * kTM * 64;
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

template <typename T, typename TO>
rtoss_status launch_typed(const rtoss_wdesc& d, const ConvParams& c, const char* section, const void* x, void* y, hipStream_t s)
{
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
