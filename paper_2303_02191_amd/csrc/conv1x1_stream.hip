// 1x1 pattern-pruned convolution as a streaming kernel with register-resident weights
// (fp16 / bf16, fp32 accumulate), and the packer that writes its weight fragments.
//
// Section IV.D prunes a 1x1 layer by cutting the flattened [Co][Ci] weight matrix into groups
// of 9 and keeping k weights per group; the pruned layer is the GEMM
//     Y[p][co] = sum_ci W'[co][ci] * X[p][ci]          (p runs over all N*H*W positions).
// The k-of-9 sparsity has no shape a matrix instruction could skip, and the layer moves every
// activation byte once for at most Ci*k/9 multiply-adds per output: it is bound by HBM, not by
// arithmetic.  So the weights are expanded to zero-filled dense fragments and the kernel is
// organised around the activation stream:
//   * Workgroups are persistent.  Each owns one block of output channels and a contiguous range
//     of positions, and every wave loads its share of the weight fragments into registers once
//     (at most 32 fragments = 128 registers), so the K loop reads weights from nowhere.
//   * Activations arrive through a ring of 3 LDS buffers filled by global -> LDS copies.  A
//     buffer holds PB positions (16 per wave along positions) x all Ci channels, laid out
//     [32-channel stage][position][64 bytes] with the four 16-byte chunks of a position
//     XOR-swizzled by (position / 2) % 4: conflict-free 16-byte operand reads without padding.
//   * A fifth wave is the producer: it issues every copy (but for the first two buffers of a
//     workgroup, which the consumers fetch while they would otherwise idle) and nothing else, so its count of
//     outstanding memory operations counts copies only and "buffer b has landed" is an exact
//     counted wait (the four consumer waves also store outputs, which would share the counter).
//     One barrier per buffer hands a filled buffer to the consumers and a drained one back.
//   * Output rows are stored straight from the accumulators.  The packer assigns output channels
//     to matrix rows so that a lane's 4*MT accumulator values are consecutive channels: row
//     4q+i of the wave's m-th fragment is channel 4*MT*q + 4*m + i of the wave's slice, and the
//     four lane quarters of a position together write one contiguous run of 16*MT channels.
//
// Operand layout of v_mfma_f32_16x16x32 (wave64; r = lane % 16, q = lane / 16): A lane holds
// row r, K = 8q..8q+7; B lane holds column r, K = 8q..8q+7; D lane holds column r, rows 4q..4q+3.
#include <algorithm>

#include "common.h"
#include "dtypes.h"
#include "epilogue.h"
#include "mma.h"
#include "pack_live.h"

namespace rtoss {

namespace {

constexpr int kFrag = 1024;  // one A fragment: 64 lanes x 16 bytes = 16 output channels x 32 input channels
constexpr int kHeadBuffers = 2;  // buffers of a workgroup's range that the consumer waves copy themselves

// Shape plan, a function of KS = Ci / 32 (1, 2, 4 ... 32) and of WM, the number of waves a
// workgroup spreads over output channels (the other 4 / WM spread over positions).
template <int KS, int WM> struct Plan {
    static constexpr int MT = KS <= 8 ? 4 : (KS == 16 ? 2 : 1);  // fragments per wave along output channels
    static constexpr int WN = 4 / WM;
    // 16-position blocks per wave and buffer: one.  (Buffers of up to four blocks per wave, 16 KB for most shapes,
    // measured slower on a 57-layer model, 0.906 against 0.892-0.895 ms: small buffers mean small workgroups in LDS,
    // more of them per compute unit and more independent streams in flight.)
    static constexpr int NB = 1;
    static constexpr int PB = 16 * NB * WN;                        // positions per buffer
    static constexpr int BUF = PB * KS * 64;                       // bytes per buffer
    static constexpr int COPIES = PB * KS / 16;                    // copy instructions (64 lanes x 16 B) per buffer
    static constexpr int SPAN = 16 * MT * WM;                      // output channels per workgroup
    // Ring depth: three buffers (one being multiplied, one landing, one being refilled).  The 6-bit counter of
    // outstanding copies would allow up to six for most shapes; measured on a 57-layer model, the shallow ring is
    // faster (0.900 vs 0.907 ms with four and 0.915 ms with up to six buffers): its 48 KB let three workgroups share a
    // compute unit, and their producers together keep more copies in flight than one deep ring can count.
    static constexpr int RING = 3;
    static_assert(COPIES >= 1 && COPIES * 16 == PB * KS, "a buffer is a whole number of copy instructions");
    static_assert(RING >= 3 && (RING - 2) * COPIES < 64, "outstanding copies must fit the counter");
};

// s_waitcnt immediate that waits for the vector-memory counter only (6 bits, split 4 + 2)
__device__ __host__ constexpr int vmcnt_imm(int n) { return 0x0f70 | (n & 15) | ((n >> 4) << 14); }

// wait until at most `later` buffers (1 .. MAXL) of COPIES copy instructions each are outstanding
template <int MAXL, int COPIES> __device__ __forceinline__ void wait_tail(int64_t later)
{
    if constexpr (MAXL >= 1) {
        if (later == MAXL) __builtin_amdgcn_s_waitcnt(vmcnt_imm(MAXL * COPIES));
        else wait_tail<MAXL - 1, COPIES>(later);
    } else {
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    }
}

inline int mt_of(int KS) { return KS <= 8 ? 4 : (KS == 16 ? 2 : 1); }
inline int wm_of(int KS, int Co)
{
    const int tiles = (Co + 15) / 16, groups = (tiles + mt_of(KS) - 1) / mt_of(KS);
    const int by_channels = groups >= 3 ? 4 : groups;  // 1, 2 or 4 waves along output channels
    // deep layers: fewer waves along positions, so that a buffer (16 positions per such wave x Ci) stays <= 32 KB
    const int by_depth = KS >= 32 ? 4 : (KS == 16 ? 2 : 1);
    return std::max(by_channels, by_depth);
}
inline int co_blocks_of(int KS, int Co)
{
    const int span = 16 * mt_of(KS) * wm_of(KS, Co);
    return (Co + span - 1) / span;
}
inline size_t frag_bytes(const rtoss_wdesc& d)
{
    const int KS = d.Ci / 32;
    return (size_t)co_blocks_of(KS, d.Co) * wm_of(KS, d.Co) * mt_of(KS) * KS * kFrag;
}
inline size_t zero_bytes(const rtoss_wdesc& d) { return align_up((size_t)2 * d.Ci + 16, 256); }

// Fragment order: [channel block][wave slice wm][fragment m][stage s][lane].
struct StreamPackArgs {
    const void* w;
    const uint8_t* idx;
    char* out;
    int Co, Ci, KS, MT, WM, zero_items;
    int64_t G, total_items;
    LiveJob job;
};

// One block of 256 items of one layer (`block` counts from the layer's first block).
template <typename T>
__device__ __forceinline__ void pack_stream1x1_body(const StreamPackArgs& a, const Dict& dict, int block)
{
    const T* __restrict__ w = (const T*)a.w;
    const uint8_t* __restrict__ idx = a.idx;
    char* __restrict__ out = a.out;
    const int Co = a.Co, Ci = a.Ci, KS = a.KS, MT = a.MT, WM = a.WM, zero_items = a.zero_items;
    const int64_t G = a.G, total_items = a.total_items;
    const LiveJob job = a.job;
    __shared__ uint16_t masks[256];
    masks[threadIdx.x] = dict.mask[threadIdx.x];
    __syncthreads();
    if (block < job.blocks) {  // the first blocks write the blob's public section
        pack_live_block<T>(w, idx, masks, dict.k, job, block);
        return;
    }
    const int64_t item = (int64_t)(block - job.blocks) * 256 + threadIdx.x;
    if (item >= total_items) {
        if (item < total_items + zero_items) *(u32x4*)(out + total_items * 16 + (item - total_items) * 16) = u32x4{0, 0, 0, 0};
        return;
    }
    const int lane = (int)(item % 64);
    int64_t f = item / 64;
    const int s = (int)(f % KS);
    f /= KS;
    const int m = (int)(f % MT);
    f /= MT;
    const int wm = (int)(f % WM);
    const int cb = (int)(f / WM);
    const int r = lane % 16, q = lane / 16;
    const int co = cb * (16 * MT * WM) + wm * (16 * MT) + (r / 4) * (4 * MT) + 4 * m + (r % 4);
    uint16_t v[8];
    for (int j = 0; j < 8; ++j) {
        const int ci = 32 * s + 8 * q + j;
        v[j] = 0;
        if (co < Co) {
            // element e of the flattened matrix sits in group e/9 at tap e%9 (groups may straddle rows)
            const int64_t e = (int64_t)co * Ci + ci;
            const int64_t g = e / 9;
            const int t = (int)(e - 9 * g);
            if (g < G && ((masks[idx[g]] >> t) & 1u)) v[j] = __builtin_bit_cast(uint16_t, w[e]);
        }
    }
    u32x4 pk;
    pk.x = v[0] | ((uint32_t)v[1] << 16);
    pk.y = v[2] | ((uint32_t)v[3] << 16);
    pk.z = v[4] | ((uint32_t)v[5] << 16);
    pk.w = v[6] | ((uint32_t)v[7] << 16);
    *(u32x4*)(out + item * 16) = pk;
}

template <typename T>
__global__ __launch_bounds__(256) void pack_stream1x1_kernel(StreamPackArgs a, Dict dict)
{
    pack_stream1x1_body<T>(a, dict, (int)blockIdx.x);
}

struct StreamPackBatch {
    StreamPackArgs a[kPackBatchMax];
    int first_block[kPackBatchMax + 1];
    int n;
};

template <typename T>
__global__ __launch_bounds__(256) void pack_stream1x1_batch_kernel(StreamPackBatch b, Dict dict)
{
    const int t = batch_entry(b, (int)blockIdx.x);  // block-uniform
    pack_stream1x1_body<T>(b.a[t], dict, (int)blockIdx.x - b.first_block[t]);
}


template <typename T, typename TO, int KS, int WM>
__global__ __launch_bounds__(320) void conv1x1_stream_kernel(const T* __restrict__ x, TO* __restrict__ y,
                                                             const char* __restrict__ wfrag, const char* __restrict__ zeros,
                                                             int64_t P, int Co, int co_blocks, int64_t nbuf, int wgs_per_cb,
                                                             int total_wgs, int work_per_xcd, Epilogue ep)
{
    using PL = Plan<KS, WM>;
    constexpr int MT = PL::MT, WN = PL::WN, NB = PL::NB, PB = PL::PB, BUF = PL::BUF, COPIES = PL::COPIES, RING = PL::RING;
    constexpr int Ci = 32 * KS;
    extern __shared__ __attribute__((aligned(16))) char smem[];  // RING buffers

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // XCD-contiguous order: the channel blocks of one position range, and neighbouring ranges, share an L2
    const int work = (blockIdx.x % 8) * work_per_xcd + blockIdx.x / 8;
    if (work >= total_wgs) return;
    const int cb = work % co_blocks, part = work / co_blocks;
    const int64_t b0 = nbuf * part / wgs_per_cb, b1 = nbuf * (part + 1) / wgs_per_cb;
    if (b0 >= b1) return;

    if (wave == 4) {
        // ---- producer wave: all global -> LDS copies of the workgroup.  It issues nothing else, so its
        // memory counter counts copies only and "at most (RING-2) buffers outstanding" is exact. ----
        int src_off[COPIES];  // byte offset from the buffer's first position of the chunk this lane fills
        int src_pos[COPIES];
#pragma unroll
        for (int k = 0; k < COPIES; ++k) {
            const int c = k * 64 + lane;
            const int s = c / (PB * 4), rem = c % (PB * 4);
            const int pos = rem >> 2, q = (rem & 3) ^ ((pos >> 1) & 3);
            src_pos[k] = pos;
            src_off[k] = (pos * Ci + s * 32 + q * 8) * 2;
        }
        auto issue_buffer = [&](int64_t b, int slot) {
            const int64_t p0 = b * PB;
            const char* base = (const char*)x + p0 * (Ci * 2);
            char* dst = smem + slot * BUF;
            if (p0 + PB <= P) {
#pragma unroll
                for (int k = 0; k < COPIES; ++k) copy16_to_lds(base + src_off[k], dst + k * 1024);
            } else {  // ragged last buffer: positions past the end read the packer's block of zeros
#pragma unroll
                for (int k = 0; k < COPIES; ++k)
                    copy16_to_lds(p0 + src_pos[k] < P ? base + src_off[k] : zeros, dst + k * 1024);
            }
        };
        // (the first kHeadBuffers buffers are copied by the consumer waves, see below)
        for (int i = kHeadBuffers; i < RING - 1; ++i)
            if (b0 + i < b1) issue_buffer(b0 + i, i);
        int slot = 0;
        for (int64_t b = b0; b < b1; ++b) {
            asm volatile("" ::: "memory");
            if (b - b0 >= kHeadBuffers) {
                // buffer b has landed once no more copies are outstanding than were issued after it
                const int64_t later = std::min<int64_t>(b1 - 1 - b, RING - 2);
                if (later >= RING - 2) __builtin_amdgcn_s_waitcnt(vmcnt_imm((RING - 2) * COPIES));
                else if (later == 0) __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
                else wait_tail<RING - 3, COPIES>(later);
            }
            __builtin_amdgcn_s_barrier();  // consumers may read buffer b; they are done with the slot refilled next
            asm volatile("" ::: "memory");
            if (b + RING - 1 < b1) issue_buffer(b + RING - 1, (slot + RING - 1) % RING);
            slot = slot + 1 == RING ? 0 : slot + 1;
        }
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
        return;
    }

    // ---- consumer waves ----
    const int wm = wave % WM, wn = wave / WM;
    // this wave's weight fragments, resident for the whole kernel
    u32x4 a[MT][KS];
    {
        const char* af = wfrag + ((int64_t)(cb * WM + wm) * MT * KS) * kFrag + lane * 16;
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int s = 0; s < KS; ++s) a[m][s] = *(const u32x4*)(af + (m * KS + s) * kFrag);
    }
    // Start-up: one wave needs about 70 cycles per copy instruction, so a producer that fills the ring alone
    // delivers the first buffer late.  The four consumer waves, idle until then, issue the copies of the
    // first kHeadBuffers buffers (every fourth copy instruction each), and wait for them together with
    // their weight fragments before the first barrier.
    for (int i = 0; i < kHeadBuffers; ++i) {
        const int64_t bb = b0 + i;
        if (bb >= b1) break;
        const int64_t p0 = bb * PB;
        const char* base = (const char*)x + p0 * (Ci * 2);
        char* dst = smem + i * BUF;
#pragma unroll
        for (int t = 0; t < (COPIES + 3) / 4; ++t) {
            const int k = wave + 4 * t;  // wave-uniform
            if (k >= COPIES) break;
            const int c = k * 64 + lane;
            const int st = c / (PB * 4), rem = c % (PB * 4);
            const int pos = rem >> 2, q = (rem & 3) ^ ((pos >> 1) & 3);
            copy16_to_lds(p0 + pos < P ? base + (pos * Ci + st * 32 + q * 8) * 2 : zeros, dst + k * 1024);
        }
    }
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    asm volatile("" ::: "memory");

    const int nn = lane & 15, qq = lane >> 4;
    // operand read offset within a buffer for stage 0, block 0 (the swizzle depends on nn only)
    const int x_lane = (wn * 16 + nn) * 64 + ((qq ^ ((nn >> 1) & 3)) * 16);
    const int co_lane = cb * PL::SPAN + wm * (16 * MT) + 4 * MT * qq;  // first of this lane's 4*MT channels
    constexpr int EB = (int)sizeof(TO);

    int slot = 0;
    for (int64_t b = b0; b < b1; ++b) {
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): this wave's reads of the previous buffer are complete
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");

        const char* X = smem + slot * BUF + x_lane;
        f32x4 acc[MT][NB];
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int j = 0; j < NB; ++j) acc[m][j] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < KS; ++s)
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                const u32x4 bv = *(const u32x4*)(X + (s * PB + 16 * WN * j) * 64);
#pragma unroll
                for (int m = 0; m < MT; ++m) acc[m][j] = Dense16<T>::mma(a[m][s], bv, acc[m][j]);
            }

        // ---- store: this lane's 4*MT consecutive channels of position nn of each of its blocks ----
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            const int64_t p = b * PB + 16 * (wn + WN * j) + nn;
            if (p >= P || co_lane >= Co) continue;  // Co is a multiple of 16 and the run is 16-aligned: all in or all out
            TO* yp = y + p * ep.ldy + co_lane;
            float v[4 * MT];
#pragma unroll
            for (int m = 0; m < MT; ++m)
#pragma unroll
                for (int e = 0; e < 4; ++e) v[4 * m + e] = acc[m][j][e];
            epi_scale_bias_act<4 * MT>(v, ep, co_lane);
            epi_residual<TO, 4 * MT>(v, ep, p, co_lane);
            if constexpr (EB == 4) {
#pragma unroll
                for (int g = 0; g < MT; ++g) *(f32x4*)(yp + 4 * g) = f32x4{v[4 * g], v[4 * g + 1], v[4 * g + 2], v[4 * g + 3]};
            } else if constexpr (MT == 1) {
                uint2 o;
                o.x = pack2_from_f32<TO>(v[0], v[1]);
                o.y = pack2_from_f32<TO>(v[2], v[3]);
                *(uint2*)yp = o;
            } else {
#pragma unroll
                for (int g = 0; g < MT / 2; ++g) {
                    u32x4 o;
                    o.x = pack2_from_f32<TO>(v[8 * g + 0], v[8 * g + 1]);
                    o.y = pack2_from_f32<TO>(v[8 * g + 2], v[8 * g + 3]);
                    o.z = pack2_from_f32<TO>(v[8 * g + 4], v[8 * g + 5]);
                    o.w = pack2_from_f32<TO>(v[8 * g + 6], v[8 * g + 7]);
                    *(u32x4*)(yp + 8 * g) = o;
                }
            }
        }
        slot = slot + 1 == RING ? 0 : slot + 1;
    }
}

template <typename T, typename TO, int KS, int WM>
rtoss_status launch_plan(const rtoss_wdesc& d, const ConvParams& c, const char* wfrag, const void* x, void* y, hipStream_t s)
{
    using PL = Plan<KS, WM>;
    const int64_t P = (int64_t)c.N * c.H * c.W;
    const int64_t nbuf = (P + PL::PB - 1) / PL::PB;
    const int co_blocks = co_blocks_of(KS, d.Co);
    const size_t smem = (size_t)PL::RING * PL::BUF;
    auto kern = conv1x1_stream_kernel<T, TO, KS, WM>;
    static LaunchOnce lds_once;  // per instantiation
    if (rtoss_status st = ensure_dynamic_lds((const void*)kern, smem, lds_once, "conv1x1 shared memory attribute")) return st;
    // Persistent workgroups: as many as are resident at once, but no fewer than 2 buffers each: every
    // workgroup loads its weight fragments once, which for deep layers is more bytes than a buffer.
    // (workgroups per compute unit depend on the instantiation's registers and LDS only: asked once; the
    // number of compute units is the current device's)
    static std::atomic<int> per_cu_cached{0};  // per instantiation
    int per_cu = per_cu_cached.load(std::memory_order_relaxed);
    if (per_cu == 0) {
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void*)kern, 320, smem) != hipSuccess || per_cu < 1) per_cu = 1;
        per_cu_cached.store(per_cu, std::memory_order_relaxed);
    }
    DeviceInfo dev;
    if (rtoss_status st = current_device(&dev)) return st;
    const int resident = std::max(8, dev.cus) * per_cu;
    const int64_t by_work = std::max<int64_t>(1, (nbuf + 1) / 2);
    const int wgs_per_cb = (int)std::max<int64_t>(1, std::min<int64_t>(by_work, resident / co_blocks));
    const int total = wgs_per_cb * co_blocks;
    const int work_per_xcd = (total + 7) / 8;
    if (P * d.Ci * 2 / PL::PB > 0x7fffffffffffll || nbuf > 0x7fffffff) return fail(RTOSS_ESHAPE, "conv1x1: too many positions");
    dim3 grid((unsigned)(work_per_xcd * 8)), block(320);
    kern<<<grid, block, smem, s>>>((const T*)x, (TO*)y, wfrag, wfrag + frag_bytes(d), P, d.Co, co_blocks, nbuf, wgs_per_cb,
                                   total, work_per_xcd, c.ep);
    return check_hip(hipGetLastError(), "conv1x1 stream launch");
}

template <typename T, typename TO, int KS>
rtoss_status launch_ks(const rtoss_wdesc& d, const ConvParams& c, const char* wfrag, const void* x, void* y, hipStream_t s)
{
    const int wm = wm_of(KS, d.Co);
    if constexpr (KS <= 8)
        if (wm == 1) return launch_plan<T, TO, KS, 1>(d, c, wfrag, x, y, s);
    if constexpr (KS <= 16)
        if (wm == 2) return launch_plan<T, TO, KS, 2>(d, c, wfrag, x, y, s);
    return launch_plan<T, TO, KS, 4>(d, c, wfrag, x, y, s);
}

template <typename T, typename TO>
rtoss_status launch_typed(const rtoss_wdesc& d, const ConvParams& c, const char* wfrag, const void* x, void* y, hipStream_t s)
{
    switch (d.Ci / 32) {
    case 1: return launch_ks<T, TO, 1>(d, c, wfrag, x, y, s);
    case 2: return launch_ks<T, TO, 2>(d, c, wfrag, x, y, s);
    case 4: return launch_ks<T, TO, 4>(d, c, wfrag, x, y, s);
    case 8: return launch_ks<T, TO, 8>(d, c, wfrag, x, y, s);
    case 16: return launch_ks<T, TO, 16>(d, c, wfrag, x, y, s);
    case 32: return launch_ks<T, TO, 32>(d, c, wfrag, x, y, s);
    }
    return fail(RTOSS_ESHAPE, "conv1x1 stream: unsupported input channel count %d", d.Ci);
}

}  // namespace

// ---- host-visible entry points of this file ----

bool stream1x1_shape_ok(const rtoss_wdesc& d)
{
    const int KS = d.Ci / 32;
    return d.ksize == 1 && (d.dt == RTOSS_F16 || d.dt == RTOSS_BF16) && d.Ci % 32 == 0 && d.Co % 16 == 0 && KS >= 1 &&
           KS <= 32 && (KS & (KS - 1)) == 0;
}

size_t stream1x1_section_bytes(const rtoss_wdesc& d) { return frag_bytes(d) + zero_bytes(d); }

static StreamPackArgs stream_pack_args(const rtoss_wdesc& d, const void* w, const uint8_t* idx, void* section,
                                       void* live_values, uint8_t* live_idx, int* blocks)
{
    StreamPackArgs a;
    a.w = w;
    a.idx = idx;
    a.out = (char*)section;
    a.Co = d.Co;
    a.Ci = d.Ci;
    a.KS = d.Ci / 32;
    a.MT = mt_of(a.KS);
    a.WM = wm_of(a.KS, d.Co);
    a.G = (int64_t)d.Co * d.Ci / 9;
    a.total_items = (int64_t)(frag_bytes(d) / 16);
    a.zero_items = (int)(zero_bytes(d) / 16);
    a.job = make_live_job(live_values, live_idx, a.G);
    *blocks = (int)(a.job.blocks + (a.total_items + a.zero_items + 255) / 256);
    return a;
}

rtoss_status launch_pack_stream1x1(const rtoss_wdesc& d, const void* w, const uint8_t* idx, const Dict& dict, void* section,
                                   void* live_values, uint8_t* live_idx, hipStream_t s)
{
    int blocks = 0;
    const StreamPackArgs a = stream_pack_args(d, w, idx, section, live_values, live_idx, &blocks);
    dim3 grid((unsigned)blocks), block(256);
    if (d.dt == RTOSS_F16) pack_stream1x1_kernel<f16_t><<<grid, block, 0, s>>>(a, dict);
    else pack_stream1x1_kernel<bf16_t><<<grid, block, 0, s>>>(a, dict);
    return check_hip(hipGetLastError(), "pack stream1x1 launch");
}

rtoss_status launch_pack_stream1x1_batch(const PackItem* items, int n, const Dict& dict, hipStream_t s)
{
    for (int base = 0; base < n; base += kPackBatchMax) {
        StreamPackBatch b;
        b.n = std::min(kPackBatchMax, n - base);
        int total = 0;
        for (int i = 0; i < b.n; ++i) {
            const PackItem& it = items[base + i];
            int blocks = 0;
            b.a[i] = stream_pack_args(it.d, it.w, it.idx, it.section, it.live, it.live_idx, &blocks);
            b.first_block[i] = total;
            total += blocks;
        }
        b.first_block[b.n] = total;
        dim3 grid((unsigned)total), block(256);
        if (items[base].d.dt == RTOSS_F16) pack_stream1x1_batch_kernel<f16_t><<<grid, block, 0, s>>>(b, dict);
        else pack_stream1x1_batch_kernel<bf16_t><<<grid, block, 0, s>>>(b, dict);
        if (rtoss_status st = check_hip(hipGetLastError(), "pack stream1x1 batch launch")) return st;
    }
    return RTOSS_OK;
}

rtoss_status launch_conv1x1_stream(const rtoss_wdesc& d, const ConvParams& c, const void* section, const void* x, void* y,
                                   hipStream_t s)
{
    const char* wf = (const char*)section;
    const bool f32out = c.out_dt == RTOSS_F32;
    if (d.dt == RTOSS_F16)
        return f32out ? launch_typed<f16_t, float>(d, c, wf, x, y, s) : launch_typed<f16_t, f16_t>(d, c, wf, x, y, s);
    return f32out ? launch_typed<bf16_t, float>(d, c, wf, x, y, s) : launch_typed<bf16_t, bf16_t>(d, c, wf, x, y, s);
}

}  // namespace rtoss
