// 3x3 pattern-pruned convolution in dense mode on the CDNA4 matrix cores (fp16 / bf16, fp32
// accumulate): every tap is a dense K-step and pruned weights are explicit zeros.
//
// This is the matrix-core path for dictionaries the 2-of-4 sparse instruction cannot take: a
// pattern with three or more corners, or three or more edge midpoints (4- and 5-entry connected
// patterns include such shapes: the T, the plus), or any unfiltered dictionary.  Nothing is
// skipped, so the effective rate on non-zero multiply-adds is capped at k/9 of the dense rate
// (Section II.B: zeros cost as much as any weight unless the kernel can skip them); it is also
// the "dense convolution on the same kernels" comparator when given the all-ones pattern.
//
// Workgroup = 4 waves, output tile = 64 output channels x 16x16 positions; every wave owns all
// 64 channels x 4 blocks of 4x4 positions.  K runs over stages of 32 input channels: the stage's
// 4 x 9 weight fragments (one contiguous piece of the blob) and the activation tile with halo
// (channels-last, 64-byte position pitch at stride 1 and 80 at stride 2) are copied global -> LDS, then each of the 9 taps is
// one v_mfma_f32_16x16x32 step per (channel fragment, position block) whose B operand is a plain
// 16-byte read at the tap's offset.  The LDS is single-buffered; for stride 1 two workgroups
// share a compute unit and hide each other's copy latency.
//
// Output rows are stored straight from the accumulators: the packer assigns output channels to
// matrix rows so that a lane's 16 accumulator values are 16 consecutive channels (row 4q+i of
// fragment m is channel 16q + 4m + i of the workgroup's 64), and the four lane quarters of a
// position together write 128 contiguous bytes.
//
// fp32 tensors run through the same kernel on v_mfma_f32_16x16x4_f32: a stage is then 16 input
// channels (the same 64 bytes per position), a lane's 16 bytes are 4 consecutive channels, and the
// K step of 16 channels is 4 instructions, instruction s taking element s of every lane's 16 bytes
// (the K slots of an instruction are the channels 4q + s: any assignment of channels to slots is
// valid as long as both operands use it).  Small launches use 16 channels x 4x16 positions per
// workgroup so that they still fill the chip.
//
// Operand layout of v_mfma_f32_16x16x32 (wave64; r = lane % 16, q = lane / 16): A lane holds
// row r, K = 8q..8q+7; B lane holds column r, K = 8q..8q+7; D lane holds column r, rows 4q..4q+3.
// v_mfma_f32_16x16x4_f32: A lane holds row r, K = q; B lane holds column r, K = q; same D.
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

constexpr int kFrag = 1024;            // 64 lanes x 16 bytes = 16 output channels x 32 input channels of one tap
constexpr int kTM = 4;                 // channel fragments per block of the blob (64 output channels)
constexpr int kBlockBytes = kTM * 9 * kFrag;  // weights of one (stage, channel block)
inline int stage_channels(rtoss_dtype dt) { return dt == RTOSS_F32 ? 16 : 32; }  // 64 bytes per position

inline int channel_blocks(int Co) { return (Co + 16 * kTM - 1) / (16 * kTM); }
inline size_t frag_bytes(const rtoss_wdesc& d)
{
    return (size_t)(d.Ci / stage_channels(d.dt)) * channel_blocks(d.Co) * kBlockBytes;
}
inline size_t zero_bytes(const rtoss_wdesc& d) { return align_up((size_t)elem_bytes(d.dt) * d.Ci + 16, 256); }

// Fragment order: [stage][channel block][fragment m][tap t][lane].
template <typename T>
__global__ __launch_bounds__(256) void pack_dense3x3_kernel(const T* __restrict__ w, const uint8_t* __restrict__ idx,
                                                            Dict dict, char* __restrict__ out, int Co, int Ci, int cblocks,
                                                            int64_t total_items, int zero_items, LiveJob job)
{
    __shared__ uint16_t masks[256];
    masks[threadIdx.x] = dict.mask[threadIdx.x];
    __syncthreads();
    if ((int)blockIdx.x < job.blocks) {  // the first blocks write the blob's public section
        pack_live_block<T>(w, idx, masks, dict.k, job, blockIdx.x);
        return;
    }
    const int64_t item = (int64_t)(blockIdx.x - job.blocks) * 256 + threadIdx.x;
    if (item >= total_items) {
        if (item < total_items + zero_items) *(u32x4*)(out + total_items * 16 + (item - total_items) * 16) = u32x4{0, 0, 0, 0};
        return;
    }
    const int lane = (int)(item % 64);
    int64_t f = item / 64;
    const int t = (int)(f % 9);
    f /= 9;
    const int m = (int)(f % kTM);
    f /= kTM;
    const int cb = (int)(f % cblocks);
    const int stage = (int)(f / cblocks);
    const int r = lane % 16, q = lane / 16;
    const int co = cb * (16 * kTM) + (r / 4) * 16 + 4 * m + (r % 4);
    constexpr int PER_LANE = 16 / (int)sizeof(T);  // elements in a lane's 16 bytes: 8 (16-bit) or 4 (fp32)
    T v[PER_LANE];
    for (int j = 0; j < PER_LANE; ++j) {
        const int ci = (4 * PER_LANE) * stage + PER_LANE * q + j;
        __builtin_memset(&v[j], 0, sizeof(T));
        if (co < Co) {
            const int64_t g = (int64_t)co * Ci + ci;
            if ((masks[idx[g]] >> t) & 1u) v[j] = w[g * 9 + t];
        }
    }
    u32x4 pk;
    __builtin_memcpy(&pk, v, 16);
    *(u32x4*)(out + item * 16) = pk;
}


// TM channel fragments (of the blob's blocks of 4) and RT x CT position blocks per workgroup.
template <typename T, typename TO, int S, int TM, int RT, int CT>
__global__ __launch_bounds__(256) void conv3x3_dense_kernel(const T* __restrict__ x, TO* __restrict__ y,
                                                            const char* __restrict__ wfrag, const char* __restrict__ zeros,
                                                            int H, int W, int Ci, int Co, int Ho, int Wo, int cblocks,
                                                            int tiles_c, Epilogue ep)
{
    using G = Geom<S, RT, CT>;
    constexpr int kTN = RT * CT / 4;                            // position blocks per wave
    static_assert(RT * CT % 4 == 0 && kTM % TM == 0, "four waves share the blocks; fragments split the blob's blocks evenly");
    constexpr int A_BYTES = TM * 9 * kFrag;
    constexpr int A_COPIES = A_BYTES / 1024;                    // copy instructions (64 lanes x 16 B)
    constexpr int A_PER_WAVE = (A_COPIES + 3) / 4;
    constexpr int EBI = (int)sizeof(T);                         // a stage is 64 bytes of channels per position
    constexpr int X_CHUNKS = G::x_bytes / 16;                   // including the pad chunk of every position
    constexpr int X_PER_WAVE = ((X_CHUNKS + 63) / 64 + 3) / 4;
    extern __shared__ __attribute__((aligned(16))) char smem[];  // [weights, rounded up][activations, rounded up to whole copies]
    char* lds_a = smem;
    char* lds_x = smem + A_PER_WAVE * 4096;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tile_r = blockIdx.x / tiles_c, tile_c = blockIdx.x % tiles_c;
    const int cb = blockIdx.y / (kTM / TM), m_first = (blockIdx.y % (kTM / TM)) * TM, n_img = blockIdx.z;
    const int oh0 = tile_r * G::TH, ow0 = tile_c * G::TW;
    const int ih0 = oh0 * S - 1, iw0 = ow0 * S - 1;
    const int stages = Ci / (64 / EBI);

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
        x_ptr[k] = inside ? (const char*)x + ((((int64_t)n_img * H + ih) * W + iw) * Ci + q * (16 / EBI)) * EBI : zeros;
    }
    const char* a_src = wfrag + (int64_t)cb * kBlockBytes + m_first * 9 * kFrag + lane * 16;
    const int64_t a_stage_stride = (int64_t)cblocks * kBlockBytes;

    const int nn = lane & 15, qq = lane >> 4;
    const int pr = nn >> 2, pc = nn & 3;
    int xb[kTN];  // LDS byte offset of this lane's position in each of its blocks, tap (0,0), its 8 channels
#pragma unroll
    for (int j = 0; j < kTN; ++j) {
        const int blk = wave * kTN + j;
        xb[j] = (((4 * (blk / CT) + pr) * S) * G::LW + (4 * (blk % CT) + pc) * S) * G::kPos + qq * 16;
    }

    // The accumulators are never cleared: the first tap of the first stage multiplies onto the
    // instruction's constant-zero C operand.  (Clearing them in the accumulation registers costs about
    // 18 cycles per register in front of the next matrix instruction.)
    f32x4 acc[TM][kTN];
    auto run_stage = [&](auto first_tag, int stage) {
        constexpr bool FIRST = decltype(first_tag)::value;
        __syncthreads();  // everybody is done reading the previous stage
#pragma unroll
        for (int k = 0; k < A_PER_WAVE; ++k) {  // (copy slots past the fragments read the block of zeros)
            const int kk = k * 4 + wave;
            copy16_to_lds(kk < A_COPIES ? a_src + stage * a_stage_stride + kk * 1024 : zeros, lds_a + kk * 1024);
        }
#pragma unroll
        for (int k = 0; k < X_PER_WAVE; ++k) copy16_to_lds(x_ptr[k] + stage * 64, lds_x + (k * 4 + wave) * 1024);
        __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): this wave's copies have landed in LDS
        __syncthreads();                     // ... and everybody's
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            u32x4 b[kTN];
#pragma unroll
            for (int j = 0; j < kTN; ++j)
                b[j] = *(const u32x4*)(lds_x + xb[j] + ((t / 3) * G::LW + (t % 3)) * G::kPos);
#pragma unroll
            for (int m = 0; m < TM; ++m) {
                const u32x4 a = *(const u32x4*)(lds_a + (m * 9 + t) * kFrag + lane * 16);
#pragma unroll
                for (int j = 0; j < kTN; ++j)
                    acc[m][j] = Dense16<T>::mma(a, b[j], FIRST && t == 0 ? f32x4{0.f, 0.f, 0.f, 0.f} : acc[m][j]);
            }
        }
    };
    run_stage(std::true_type{}, 0);
    for (int stage = 1; stage < stages; ++stage) run_stage(std::false_type{}, stage);

    // ---- store: 4*TM consecutive channels of this lane's position in each of its blocks ----
    const int co_lane = cb * (16 * kTM) + 16 * qq + 4 * m_first;
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
        } else if constexpr (TM == 1) {
            uint2 o;
            o.x = pack2_from_f32<TO>(v[0], v[1]);
            o.y = pack2_from_f32<TO>(v[2], v[3]);
            *(uint2*)yp = o;
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

template <typename T, typename TO, int S, int TM, int RT, int CT>
rtoss_status launch_shape(const rtoss_wdesc& d, const ConvParams& c, const char* wfrag, const void* x, void* y, hipStream_t s)
{
    using G = Geom<S, RT, CT>;
    const int Ho = (c.H + 2 - 3) / S + 1, Wo = (c.W + 2 - 3) / S + 1;
    const int tiles_r = (Ho + G::TH - 1) / G::TH, tiles_c = (Wo + G::TW - 1) / G::TW;
    const int cblocks = channel_blocks(d.Co);
    constexpr int x_copies_per_wave = ((G::x_bytes / 16 + 63) / 64 + 3) / 4;
    constexpr int a_copies_per_wave = (TM * 9 + 3) / 4;
    const size_t smem = (size_t)(a_copies_per_wave + x_copies_per_wave) * 4096;
    auto kern = conv3x3_dense_kernel<T, TO, S, TM, RT, CT>;
    static LaunchOnce lds_once;  // per instantiation
    if (rtoss_status st = ensure_dynamic_lds((const void*)kern, smem, lds_once, "conv3x3 dense shared memory attribute")) return st;
    const int ygrid = cblocks * (kTM / TM);
    if (c.N > 65535 || ygrid > 65535) return fail(RTOSS_ESHAPE, "conv: batch or channel count too large");
    dim3 grid((unsigned)(tiles_r * tiles_c), (unsigned)ygrid, (unsigned)c.N), block(256);
    kern<<<grid, block, smem, s>>>((const T*)x, (TO*)y, wfrag, wfrag + frag_bytes(d), c.H, c.W, d.Ci, d.Co, Ho, Wo, cblocks,
                                   tiles_c, c.ep);
    return check_hip(hipGetLastError(), "conv3x3 dense launch");
}

template <typename T, typename TO, int S>
rtoss_status launch_stride(const rtoss_wdesc& d, const ConvParams& c, const char* wfrag, const void* x, void* y, hipStream_t s)
{
    // 64 channels x 16x16 positions per workgroup; launches that would not fill the chip that way take
    // 16 channels x 4x16 positions (16 times as many workgroups).
    const int Ho = (c.H + 2 - 3) / S + 1, Wo = (c.W + 2 - 3) / S + 1;
    const int64_t big = (int64_t)((Ho + 15) / 16) * ((Wo + 15) / 16) * channel_blocks(d.Co) * c.N;
    if (big < 256) return launch_shape<T, TO, S, 1, 1, 4>(d, c, wfrag, x, y, s);
    return launch_shape<T, TO, S, 4, 4, 4>(d, c, wfrag, x, y, s);
}

template <typename T, typename TO>
rtoss_status launch_typed(const rtoss_wdesc& d, const ConvParams& c, const char* wfrag, const void* x, void* y, hipStream_t s)
{
    if (c.stride == 1) return launch_stride<T, TO, 1>(d, c, wfrag, x, y, s);
    return launch_stride<T, TO, 2>(d, c, wfrag, x, y, s);
}

}  // namespace

// ---- host-visible entry points of this file ----

bool dense3x3_shape_ok(const rtoss_wdesc& d)
{
    return d.ksize == 3 && d.Ci % stage_channels(d.dt) == 0 && d.Co % 16 == 0;
}

size_t dense3x3_section_bytes(const rtoss_wdesc& d) { return frag_bytes(d) + zero_bytes(d); }

rtoss_status launch_pack_dense3x3(const rtoss_wdesc& d, const void* w, const uint8_t* idx, const Dict& dict, void* section,
                                  void* live_values, uint8_t* live_idx, hipStream_t s)
{
    const LiveJob job = make_live_job(live_values, live_idx, (int64_t)d.Co * d.Ci);
    const int cblocks = channel_blocks(d.Co);
    const int64_t items = (int64_t)(frag_bytes(d) / 16);
    const int zero_items = (int)(zero_bytes(d) / 16);
    dim3 grid((unsigned)(job.blocks + (items + zero_items + 255) / 256)), block(256);
    if (d.dt == RTOSS_F16)
        pack_dense3x3_kernel<f16_t><<<grid, block, 0, s>>>((const f16_t*)w, idx, dict, (char*)section, d.Co, d.Ci, cblocks, items, zero_items, job);
    else if (d.dt == RTOSS_BF16)
        pack_dense3x3_kernel<bf16_t><<<grid, block, 0, s>>>((const bf16_t*)w, idx, dict, (char*)section, d.Co, d.Ci, cblocks, items, zero_items, job);
    else
        pack_dense3x3_kernel<float><<<grid, block, 0, s>>>((const float*)w, idx, dict, (char*)section, d.Co, d.Ci, cblocks, items, zero_items, job);
    return check_hip(hipGetLastError(), "pack dense3x3 launch");
}

rtoss_status launch_conv3x3_dense(const rtoss_wdesc& d, const ConvParams& c, const void* section, const void* x, void* y,
                                  hipStream_t s)
{
    const char* wf = (const char*)section;
    const bool f32out = c.out_dt == RTOSS_F32;
    if (d.dt == RTOSS_F32) return launch_typed<float, float>(d, c, wf, x, y, s);
    if (d.dt == RTOSS_F16)
        return f32out ? launch_typed<f16_t, float>(d, c, wf, x, y, s) : launch_typed<f16_t, f16_t>(d, c, wf, x, y, s);
    return f32out ? launch_typed<bf16_t, float>(d, c, wf, x, y, s) : launch_typed<bf16_t, bf16_t>(d, c, wf, x, y, s);
}

}  // namespace rtoss
