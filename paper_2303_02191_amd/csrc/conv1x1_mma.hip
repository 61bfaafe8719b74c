// 1x1 pattern-pruned convolution on the CDNA4 matrix cores (fp16 / bf16, fp32 accumulate),
// and the packer that writes its weight fragments: the general kernel, for any input channel
// count that is a multiple of 32.  (Channel counts of the form 32 * 2^n up to 1024 take the
// streaming kernel with register-resident weights instead.)
//
// Section IV.D prunes a 1x1 layer by cutting the flattened [Co][Ci] weight matrix into groups
// of 9 and keeping k weights per group, so the pruned layer is a GEMM
//     Y[p][co] = sum_ci W'[co][ci] * X[p][ci]          (p runs over all N*H*W positions)
// whose weight matrix has k-of-9 sparsity along its flattened axis.  That sparsity has no
// structure a matrix instruction could skip (groups straddle rows and have no 2-of-4 shape),
// and the layer is bound by HBM traffic anyway: activations in, activations out, every byte
// once.  So the weights are expanded to zero-filled dense fragments (they are tiny and stay in
// L2), and the kernel is built to stream activations: channels-last rows are contiguous, a
// workgroup owns 128 consecutive positions x up to 128 output channels, and K runs over stages
// of 32 input channels through a 5-deep ring of LDS buffers filled by global -> LDS copies four
// stages ahead (an HBM-bound kernel lives on bytes in flight: two resident workgroups per CU x
// four stages x 8 KB of activations).  Activation rows sit in LDS at a 64-byte pitch with their
// four 16-byte chunks XOR-swizzled by (position / 2) % 4, which makes the 16-byte operand reads
// of 8 neighbouring positions hit 8 different bank groups without any padding.
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

constexpr int kFrag = 1024;      // one A fragment: 64 lanes x 16 bytes = 16 output channels x 32 input channels
constexpr int kTilePos = 128;    // positions per workgroup
constexpr int kRing = 5;

inline int padded_tiles(int Co) { return ((Co + 15) / 16 + 7) / 8 * 8; }
inline size_t frag_bytes(const rtoss_wdesc& d) { return (size_t)(d.Ci / 32) * padded_tiles(d.Co) * kFrag; }
inline size_t zero_bytes(const rtoss_wdesc& d) { return align_up((size_t)2 * d.Ci + 16, 256); }

template <typename T>
__global__ __launch_bounds__(256) void pack_dense1x1_kernel(const T* __restrict__ w, const uint8_t* __restrict__ idx,
                                                            Dict dict, char* __restrict__ out, int Co, int Ci, int m_tiles,
                                                            int64_t G, int64_t total_items, int zero_items, LiveJob job)
{
    __shared__ uint16_t masks[256];
    masks[threadIdx.x] = dict.mask[threadIdx.x];
    __syncthreads();
    if ((int)blockIdx.x < job.blocks) {  // the first blocks write the blob's public section
        pack_live_block<T>(w, idx, masks, dict.k, job, blockIdx.x);
        return;
    }
    const int64_t item = (int64_t)(blockIdx.x - job.blocks) * 256 + threadIdx.x;  // (stage, m_tile, lane)
    if (item >= total_items) {
        if (item < total_items + zero_items) *(u32x4*)(out + total_items * 16 + (item - total_items) * 16) = u32x4{0, 0, 0, 0};
        return;
    }
    const int lane = (int)(item % 64);
    const int64_t tile = item / 64;
    const int mt = (int)(tile % m_tiles), cb = (int)(tile / m_tiles);
    const int co = 16 * mt + (lane % 16), q = lane / 16;
    uint16_t v[8];
    for (int j = 0; j < 8; ++j) {
        const int ci = 32 * cb + 8 * q + j;
        v[j] = 0;
        if (co < Co && ci < Ci) {
            // element f of the flattened matrix sits in group f/9 at tap f%9 (groups may straddle rows)
            const int64_t f = (int64_t)co * Ci + ci;
            const int64_t g = f / 9;
            const int t = (int)(f - 9 * g);
            if (g < G && ((masks[idx[g]] >> t) & 1u)) v[j] = __builtin_bit_cast(uint16_t, w[f]);
        }
    }
    u32x4 pk;
    pk.x = v[0] | ((uint32_t)v[1] << 16);
    pk.y = v[2] | ((uint32_t)v[3] << 16);
    pk.z = v[4] | ((uint32_t)v[5] << 16);
    pk.w = v[6] | ((uint32_t)v[7] << 16);
    *(u32x4*)(out + item * 16) = pk;
}

template <typename T, typename TO, int TM>
__global__ __launch_bounds__(256) void conv1x1_mma_kernel(const T* __restrict__ x, TO* __restrict__ y,
                                                          const char* __restrict__ wfrag, const char* __restrict__ zeros,
                                                          int64_t P, int Ci, int Co, int m_tiles_total, int co_blocks,
                                                          int total_work, int work_per_xcd, Epilogue ep)
{
    constexpr int TN = 2;                                // 16-position blocks per wave
    constexpr int A_PER_WAVE = (TM + 3) / 4;             // copy instructions per wave and stage (64 lanes x 16 B each)
    constexpr int A_AREA = A_PER_WAVE * 4 * 1024;
    constexpr int X_PER_WAVE = 2;                        // 128 positions x 4 chunks = 512 chunks = 8 copies
    constexpr int X_AREA = X_PER_WAVE * 4 * 1024;
    constexpr int STAGE = A_AREA + X_AREA;
    constexpr int CPW = A_PER_WAVE + X_PER_WAVE;         // copies one wave has in flight per stage
    extern __shared__ __attribute__((aligned(16))) char smem[];  // kRing stages

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // XCD-contiguous work order (channel blocks of one position tile, and neighbouring tiles, share an L2)
    const int work = (blockIdx.x % 8) * work_per_xcd + blockIdx.x / 8;
    if (work >= total_work) return;
    const int cblk = work % co_blocks;
    const int64_t p0 = (int64_t)(work / co_blocks) * kTilePos;
    const int mt0 = cblk * TM;
    const int stages = Ci / 32;

    // ---- copy sources: every lane copies 16 bytes in every copy instruction (no branches); lanes
    // whose slot is padding read the packer's block of zeros ----
    const char* x_ptr[X_PER_WAVE];
#pragma unroll
    for (int k = 0; k < X_PER_WAVE; ++k) {
        const int c = (k * 4 + wave) * 64 + lane;          // LDS chunk this lane fills
        const int pos = c >> 2, q = (c & 3) ^ ((pos >> 1) & 3);  // ... holds channel chunk q of position pos
        const bool real = p0 + pos < P;
        x_ptr[k] = real ? (const char*)x + ((p0 + pos) * Ci + q * 8) * 2 : zeros;
    }
    const char* a_ptr[A_PER_WAVE];
#pragma unroll
    for (int k = 0; k < A_PER_WAVE; ++k) {
        const int kk = k * 4 + wave;
        a_ptr[k] = kk < TM ? wfrag + (int64_t)(mt0 + kk) * kFrag + lane * 16 : zeros;
    }
    const int64_t a_stage_stride = (int64_t)m_tiles_total * kFrag;
    auto issue_stage = [&](int stage, int buf) {
        char* base = smem + buf * STAGE;
#pragma unroll
        for (int k = 0; k < A_PER_WAVE; ++k) {
            const int kk = k * 4 + wave;
            // (the zero block is shorter than a stage stride; padding lanes re-read its start every stage)
            copy16_to_lds(kk < TM ? a_ptr[k] + stage * a_stage_stride : a_ptr[k], base + kk * 1024);
        }
#pragma unroll
        for (int k = 0; k < X_PER_WAVE; ++k) copy16_to_lds(x_ptr[k] + stage * 64, base + A_AREA + (k * 4 + wave) * 1024);
    };

    const int nn = lane & 15, qq = lane >> 4;
    f32x4 acc[TM][TN];
#pragma unroll
    for (int m = 0; m < TM; ++m)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[m][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    // kRing-1 stages are always in flight or being multiplied.  Past the end the last stage is
    // fetched again into a free buffer, so that every wave has issued exactly CPW copies per
    // stage and the wait below can count them.
    constexpr int AHEAD = kRing - 2;  // stages still in flight when a stage must have landed
    static_assert(AHEAD * CPW < 64, "outstanding copies must fit the counter");
#pragma unroll
    for (int s = 0; s < kRing - 1; ++s) issue_stage(min(s, stages - 1), s);
    int buf = 0;
    for (int s = 0; s < stages; ++s) {
        // all but the AHEAD newest stages' copies of this wave have landed ...
        // (a bare barrier: __syncthreads() would add a fence that waits for ALL outstanding copies)
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(0x0070 | ((AHEAD * CPW) & 15) | (((AHEAD * CPW) >> 4) << 14));  // + lgkmcnt(0)
        __builtin_amdgcn_s_barrier();  // ... and everybody's; everybody is done with the buffer refilled next
        asm volatile("" ::: "memory");
        issue_stage(min(s + kRing - 1, stages - 1), buf == 0 ? kRing - 1 : buf - 1);
        const char* A = smem + buf * STAGE + lane * 16;
        // position block j of this wave starts at wave*32 + 16 j; the swizzle depends on n only
        const char* X = smem + buf * STAGE + A_AREA + (wave * TN * 16 + nn) * 64 + ((qq ^ ((nn >> 1) & 3)) * 16);
        u32x4 b[TN];
#pragma unroll
        for (int j = 0; j < TN; ++j) b[j] = *(const u32x4*)(X + j * 16 * 64);
#pragma unroll
        for (int m = 0; m < TM; ++m) {
            const u32x4 a = *(const u32x4*)(A + m * kFrag);
#pragma unroll
            for (int j = 0; j < TN; ++j) Mat<T>::dense(a, b[j], acc[m][j]);
        }
        buf = buf + 1 == kRing ? 0 : buf + 1;
    }
    __builtin_amdgcn_s_waitcnt(0x0f70);  // the surplus copies have landed: LDS may be reused
    __syncthreads();
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");  // last matrix results are in the accumulators

    // ---- epilogue: transpose through LDS so that whole channel rows are written, 16 bytes per lane ----
    {
        constexpr int EB = (int)sizeof(TO);
        constexpr int HALVES = (EB == 4 && TM >= 2) ? 2 : 1;
        constexpr int TMH = TM / HALVES;
        constexpr int ROW = TMH * 16 * EB + (EB == 2 ? 8 : 16);
        static_assert(4 * 16 * TN * ROW <= kRing * STAGE, "epilogue staging must fit in the ring");
        char* stage_out = smem + wave * (16 * TN * ROW);
#pragma unroll
        for (int h = 0; h < HALVES; ++h) {
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int mm = 0; mm < TMH; ++mm) {
                    f32x4 v = acc[h * TMH + mm][j];
                    {  // output stage on this lane's 4 consecutive channels of position p_f
                        const int co4 = 16 * (mt0 + h * TMH + mm) + 4 * qq;
                        const int64_t p_f = p0 + wave * (TN * 16) + j * 16 + nn;
                        if (p_f < P && co4 < Co) {
                            float vv[4] = {v.x, v.y, v.z, v.w};
                            epi_scale_bias_act<4>(vv, ep, co4);
                            epi_residual<TO, 4>(vv, ep, p_f, co4);
                            v = f32x4{vv[0], vv[1], vv[2], vv[3]};
                        }
                    }
                    char* dst = stage_out + (j * 16 + nn) * ROW + (16 * mm + 4 * qq) * EB;
                    if constexpr (EB == 4) {
                        *(f32x4*)dst = v;
                    } else {
                        uint2 o;
                        o.x = pack2_from_f32<TO>(v.x, v.y);
                        o.y = pack2_from_f32<TO>(v.z, v.w);
                        *(uint2*)dst = o;
                    }
                }
            constexpr int CH = TMH * 16 * EB / 16;  // 16-byte chunks per row
            static_assert(64 % CH == 0, "row chunks must tile the wave");
            constexpr int POS_PER_PASS = 64 / CH;
            constexpr int PASSES = (16 * TN) / POS_PER_PASS;
            const int co_first = 16 * (mt0 + h * TMH);
#pragma unroll
            for (int ps = 0; ps < PASSES; ++ps) {
                const int pl = ps * POS_PER_PASS + lane / CH;  // position within the wave's 32
                const int chunk = lane % CH;
                const int64_t p = p0 + wave * (TN * 16) + pl;
                const int co = co_first + chunk * (16 / EB);
                const u32x4 v = *(const u32x4*)(stage_out + pl * ROW + chunk * 16);
                if (p < P && co < Co) *(u32x4*)(y + p * ep.ldy + co) = v;
            }
        }
    }
}

template <typename T, typename TO, int TM>
rtoss_status launch_tm(const rtoss_wdesc& d, const ConvParams& c, const char* wfrag, const void* x, void* y, hipStream_t s)
{
    const int64_t P = (int64_t)c.N * c.H * c.W;
    const int64_t pos_tiles = (P + kTilePos - 1) / kTilePos;
    const int co_blocks = ((d.Co + 15) / 16 + TM - 1) / TM;
    const int64_t total = pos_tiles * co_blocks;
    if (total > 0x3fffffff) return fail(RTOSS_ESHAPE, "conv1x1: too many tiles");
    const int work_per_xcd = (int)((total + 7) / 8);
    constexpr int stage_bytes = ((TM + 3) / 4) * 4096 + 2 * 4096;
    const size_t smem = (size_t)kRing * stage_bytes;
    auto kern = conv1x1_mma_kernel<T, TO, TM>;
    static LaunchOnce lds_once;  // per instantiation
    if (rtoss_status st = ensure_dynamic_lds((const void*)kern, smem, lds_once, "conv1x1 shared memory attribute")) return st;
    dim3 grid((unsigned)(work_per_xcd * 8)), block(256);
    kern<<<grid, block, smem, s>>>((const T*)x, (TO*)y, wfrag, wfrag + frag_bytes(d), P, d.Ci, d.Co, padded_tiles(d.Co),
                                   co_blocks, (int)total, work_per_xcd, c.ep);
    return check_hip(hipGetLastError(), "conv1x1 launch");
}

template <typename T, typename TO>
rtoss_status launch_typed(const rtoss_wdesc& d, const ConvParams& c, const char* wfrag, const void* x, void* y, hipStream_t s)
{
    // the fragment section is padded to a multiple of 8 channel tiles, so a block of TM <= 8 tiles never reads past it
    const int tiles = (d.Co + 15) / 16;
    if (tiles <= 2) return launch_tm<T, TO, 2>(d, c, wfrag, x, y, s);
    if (tiles <= 4) return launch_tm<T, TO, 4>(d, c, wfrag, x, y, s);
    return launch_tm<T, TO, 8>(d, c, wfrag, x, y, s);
}

}  // namespace

bool dense1x1_shape_ok(const rtoss_wdesc& d)
{
    return d.ksize == 1 && (d.dt == RTOSS_F16 || d.dt == RTOSS_BF16) && d.Ci % 32 == 0 && d.Co % 16 == 0;
}

size_t dense1x1_section_bytes(const rtoss_wdesc& d) { return frag_bytes(d) + zero_bytes(d); }

rtoss_status launch_pack_dense1x1(const rtoss_wdesc& d, const void* w, const uint8_t* idx, const Dict& dict, void* section,
                                  void* live_values, uint8_t* live_idx, hipStream_t s)
{
    const int m_tiles = padded_tiles(d.Co);
    const int64_t items = (int64_t)(d.Ci / 32) * m_tiles * 64;
    const int zero_items = (int)(zero_bytes(d) / 16);
    const int64_t G = (int64_t)d.Co * d.Ci / 9;
    const LiveJob job = make_live_job(live_values, live_idx, G);
    dim3 grid((unsigned)(job.blocks + (items + zero_items + 255) / 256)), block(256);
    if (d.dt == RTOSS_F16)
        pack_dense1x1_kernel<f16_t><<<grid, block, 0, s>>>((const f16_t*)w, idx, dict, (char*)section, d.Co, d.Ci, m_tiles, G, items, zero_items, job);
    else
        pack_dense1x1_kernel<bf16_t><<<grid, block, 0, s>>>((const bf16_t*)w, idx, dict, (char*)section, d.Co, d.Ci, m_tiles, G, items, zero_items, job);
    return check_hip(hipGetLastError(), "pack dense1x1 launch");
}

rtoss_status launch_conv1x1_mma(const rtoss_wdesc& d, const ConvParams& c, const void* section, const void* x, void* y,
                                hipStream_t s)
{
    const char* wf = (const char*)section;
    const bool f32out = c.out_dt == RTOSS_F32;
    if (d.dt == RTOSS_F16)
        return f32out ? launch_typed<f16_t, float>(d, c, wf, x, y, s) : launch_typed<f16_t, f16_t>(d, c, wf, x, y, s);
    return f32out ? launch_typed<bf16_t, float>(d, c, wf, x, y, s) : launch_typed<bf16_t, bf16_t>(d, c, wf, x, y, s);
}

}  // namespace rtoss
