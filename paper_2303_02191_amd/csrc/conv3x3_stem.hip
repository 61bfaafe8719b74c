// 3x3 convolution for very small input channel counts (the 3-channel image stem) on the dense
// matrix instruction (fp16 / bf16, fp32 accumulate).
//
// With Ci <= 3 the whole reduction, K = 9*Ci <= 27, fits one v_mfma_f32_16x16x32 step: a block
// of 16 output positions x 16 output channels is one instruction, pruned taps are explicit
// zeros in the weight fragment (there is nothing to skip in a single instruction), and the
// layer is bound by the output write.  K index k = kh*(3*Ci) + kw*Ci + ci, which is the memory
// order of a channels-last patch row, so a lane's 8 consecutive K values are short contiguous
// runs of the input tile staged in LDS.
//
// Operand layout (wave64; r = lane % 16, q = lane / 16): A lane holds row r, K = 8q..8q+7; B lane
// holds column r, K = 8q..8q+7; D lane holds column r, rows 4q..4q+3.
#include "common.h"
#include "dtypes.h"
#include "epilogue.h"
#include "mma.h"
#include "pack_live.h"

namespace rtoss {

namespace {

constexpr int kTH = 8, kTW = 32;  // output tile: 8 rows x 32 columns = 16 blocks of 16 positions


template <typename T>
__global__ __launch_bounds__(256) void pack_stem_kernel(const T* __restrict__ w, const uint8_t* __restrict__ idx, Dict dict,
                                                        char* __restrict__ out, int Co, int Ci, int m_tiles, LiveJob job)
{
    __shared__ uint16_t masks[256];
    masks[threadIdx.x] = dict.mask[threadIdx.x];
    __syncthreads();
    if ((int)blockIdx.x < job.blocks) {  // the first blocks write the blob's public section
        pack_live_block<T>(w, idx, masks, dict.k, job, blockIdx.x);
        return;
    }
    const int item = (blockIdx.x - job.blocks) * 256 + threadIdx.x;  // (m_tile, lane)
    if (item >= m_tiles * 64) return;
    const int lane = item % 64, mt = item / 64;
    // Rows are dealt over each pair of channel tiles so that the 4 + 4 accumulator values a lane holds
    // (rows 4q .. 4q+3 of both tiles) are the 8 consecutive channels 32*(mt/2) + 8q .. +7.
    const int r = lane % 16, q = lane / 16;
    const int co = 32 * (mt >> 1) + 8 * (r >> 2) + 4 * (mt & 1) + (r & 3);
    uint16_t v[8];
    for (int j = 0; j < 8; ++j) {
        const int k = 8 * q + j;
        v[j] = 0;
        if (co < Co && k < 9 * Ci) {
            const int kh = k / (3 * Ci), kw = (k % (3 * Ci)) / Ci, ci = k % Ci;
            const int t = 3 * kh + kw;
            const int64_t g9 = (int64_t)co * Ci + ci;
            if ((masks[idx[g9]] >> t) & 1u) v[j] = __builtin_bit_cast(uint16_t, w[g9 * 9 + t]);
        }
    }
    u32x4 pk;
    pk.x = v[0] | ((uint32_t)v[1] << 16);
    pk.y = v[2] | ((uint32_t)v[3] << 16);
    pk.z = v[4] | ((uint32_t)v[5] << 16);
    pk.w = v[6] | ((uint32_t)v[7] << 16);
    *(u32x4*)(out + (size_t)item * 16) = pk;
}

// Ci is a template parameter: the index arithmetic below divides by it (and by 3 * Ci) per element, which
// as run-time divisions made the kernel bound by integer ALU work.
template <typename T, typename TO, int S, int TM, int Ci>
__global__ __launch_bounds__(256, TM == 2 ? 8 : 4) void conv3x3_stem_kernel(const T* __restrict__ x, TO* __restrict__ y,
                                                           const char* __restrict__ wfrag, int H, int W, int Co,
                                                           int Ho, int Wo, int tiles_c, Epilogue ep)
{
    constexpr int IH = (kTH - 1) * S + 3, IW = (kTW - 1) * S + 3;
    constexpr int MAXROW = IW * 3 + 1;  // halves per staged row (Ci <= 3), odd pitch
    __shared__ uint16_t xs[IH * MAXROW];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tile_r = blockIdx.x / tiles_c, tile_c = blockIdx.x % tiles_c;
    const int n_img = blockIdx.y;
    const int oh0 = tile_r * kTH, ow0 = tile_c * kTW;
    const int ih0 = oh0 * S - 1, iw0 = ow0 * S - 1;
    constexpr int rowlen = IW * Ci;  // halves per row actually used

    // ---- stage the input tile (with halo, zero padded): consecutive lanes read consecutive halves; all of a
    // lane's loads are issued before the first one is used ----
    const uint16_t* xin = (const uint16_t*)x;
    constexpr int kElems = IH * rowlen, kLoads = (kElems + 255) / 256;
    uint16_t staged[kLoads];
#pragma unroll
    for (int i = 0; i < kLoads; ++i) {
        const int e = tid + 256 * i;
        const int pr = e / rowlen, off = e - pr * rowlen;
        const int ih = ih0 + pr, iw = iw0 + off / Ci;
        staged[i] = 0;
        if (e < kElems && ih >= 0 && ih < H && iw >= 0 && iw < W) staged[i] = xin[(((int64_t)n_img * H + ih) * W + iw0) * Ci + off];
    }
#pragma unroll
    for (int i = 0; i < kLoads; ++i) {
        const int e = tid + 256 * i;
        const int pr = e / rowlen, off = e - pr * rowlen;
        if (e < kElems) xs[pr * MAXROW + off] = staged[i];
    }
    // weight fragments stay in registers: TM tiles of 16 output channels
    u32x4 afrag[TM];
#pragma unroll
    for (int m = 0; m < TM; ++m) afrag[m] = *(const u32x4*)(wfrag + (m * 64 + lane) * 16);
    __syncthreads();

    const int nn = lane & 15, qq = lane >> 4;
    constexpr int k3 = 3 * Ci, K = 9 * Ci;
    // LDS offset of each of this lane's 8 K values relative to the block's first tap (same for all blocks)
    int koff[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int k = 8 * qq + j;
        const int kh = k / k3, off = k - kh * k3;
        koff[j] = k < K ? kh * MAXROW + off : -1;
    }
#pragma unroll 1
    for (int jb = 0; jb < 4; ++jb) {
        const int blk = wave * 4 + jb;            // 16 blocks: 8 rows x 2 half-rows of 16 columns
        const int r = blk >> 1, c = (blk & 1) * 16 + nn;
        uint16_t bv[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) bv[j] = koff[j] >= 0 ? xs[r * S * MAXROW + c * S * Ci + koff[j]] : (uint16_t)0;
        u32x4 b;
        b.x = bv[0] | ((uint32_t)bv[1] << 16);
        b.y = bv[2] | ((uint32_t)bv[3] << 16);
        b.z = bv[4] | ((uint32_t)bv[5] << 16);
        b.w = bv[6] | ((uint32_t)bv[7] << 16);
        const int oh = oh0 + r, ow = ow0 + c;
        const bool inside = oh < Ho && ow < Wo;
        const int64_t pos = ((int64_t)n_img * Ho + oh) * Wo + ow;
        TO* yp = y + pos * ep.ldy;
        static_assert(TM % 2 == 0, "pairs of channel tiles");
#pragma unroll
        for (int mp = 0; mp < TM; mp += 2) {
            const f32x4 d0 = Dense16<T>::mma(afrag[mp], b, f32x4{0.f, 0.f, 0.f, 0.f});
            const f32x4 d1 = Dense16<T>::mma(afrag[mp + 1], b, f32x4{0.f, 0.f, 0.f, 0.f});
            const int co = 16 * mp + 8 * qq;  // this lane's 8 consecutive channels of the pair
            if (inside && co < Co) {
                float vv[8] = {d0.x, d0.y, d0.z, d0.w, d1.x, d1.y, d1.z, d1.w};
                epi_scale_bias_act<8>(vv, ep, co);
                epi_residual<TO, 8>(vv, ep, pos, co);
                if constexpr (sizeof(TO) == 4) {
                    *(f32x4*)(yp + co) = f32x4{vv[0], vv[1], vv[2], vv[3]};
                    *(f32x4*)(yp + co + 4) = f32x4{vv[4], vv[5], vv[6], vv[7]};
                } else {
                    u32x4 o;
                    o.x = pack2_from_f32<TO>(vv[0], vv[1]);
                    o.y = pack2_from_f32<TO>(vv[2], vv[3]);
                    o.z = pack2_from_f32<TO>(vv[4], vv[5]);
                    o.w = pack2_from_f32<TO>(vv[6], vv[7]);
                    *(u32x4*)(yp + co) = o;
                }
            }
        }
    }
}

template <typename T, typename TO, int S, int TM, int Ci>
rtoss_status launch_stem_ci(const rtoss_wdesc& d, const ConvParams& c, const char* wfrag, const void* x, void* y, hipStream_t s)
{
    const int Ho = (c.H + 2 - 3) / S + 1, Wo = (c.W + 2 - 3) / S + 1;
    const int tiles_r = (Ho + kTH - 1) / kTH, tiles_c = (Wo + kTW - 1) / kTW;
    if (c.N > 65535) return fail(RTOSS_ESHAPE, "conv: batch too large");
    dim3 grid((unsigned)(tiles_r * tiles_c), (unsigned)c.N), block(256);
    conv3x3_stem_kernel<T, TO, S, TM, Ci><<<grid, block, 0, s>>>((const T*)x, (TO*)y, wfrag, c.H, c.W, d.Co, Ho, Wo, tiles_c,
                                                                 c.ep);
    return check_hip(hipGetLastError(), "conv3x3 stem launch");
}

template <typename T, typename TO, int S, int TM>
rtoss_status launch_stem(const rtoss_wdesc& d, const ConvParams& c, const char* wfrag, const void* x, void* y, hipStream_t s)
{
    if (d.Ci == 3) return launch_stem_ci<T, TO, S, TM, 3>(d, c, wfrag, x, y, s);
    if (d.Ci == 2) return launch_stem_ci<T, TO, S, TM, 2>(d, c, wfrag, x, y, s);
    return launch_stem_ci<T, TO, S, TM, 1>(d, c, wfrag, x, y, s);
}

template <typename T, typename TO>
rtoss_status launch_typed(const rtoss_wdesc& d, const ConvParams& c, const char* wfrag, const void* x, void* y, hipStream_t s)
{
    const int tiles = (d.Co + 15) / 16;
    if (c.stride == 1) {
        if (tiles <= 2) return launch_stem<T, TO, 1, 2>(d, c, wfrag, x, y, s);
        return launch_stem<T, TO, 1, 4>(d, c, wfrag, x, y, s);
    }
    if (tiles <= 2) return launch_stem<T, TO, 2, 2>(d, c, wfrag, x, y, s);
    return launch_stem<T, TO, 2, 4>(d, c, wfrag, x, y, s);
}

}  // namespace

bool stem3x3_shape_ok(const rtoss_wdesc& d)
{
    return d.ksize == 3 && (d.dt == RTOSS_F16 || d.dt == RTOSS_BF16) && d.Ci <= 3 && d.Co % 16 == 0 && d.Co <= 64;
}

size_t stem3x3_section_bytes(const rtoss_wdesc& d) { return (size_t)4 * 1024; }  // 4 tiles, unused ones zero

rtoss_status launch_pack_stem3x3(const rtoss_wdesc& d, const void* w, const uint8_t* idx, const Dict& dict, void* section,
                                 void* live_values, uint8_t* live_idx, hipStream_t s)
{
    const LiveJob job = make_live_job(live_values, live_idx, (int64_t)d.Co * d.Ci);
    dim3 grid((unsigned)(job.blocks + 1)), block(256);
    if (d.dt == RTOSS_F16)
        pack_stem_kernel<f16_t><<<grid, block, 0, s>>>((const f16_t*)w, idx, dict, (char*)section, d.Co, d.Ci, 4, job);
    else
        pack_stem_kernel<bf16_t><<<grid, block, 0, s>>>((const bf16_t*)w, idx, dict, (char*)section, d.Co, d.Ci, 4, job);
    return check_hip(hipGetLastError(), "pack stem launch");
}

rtoss_status launch_conv3x3_stem(const rtoss_wdesc& d, const ConvParams& c, const void* section, const void* x, void* y,
                                 hipStream_t s)
{
    const char* wf = (const char*)section;
    const bool f32out = c.out_dt == RTOSS_F32;
    if (d.dt == RTOSS_F16)
        return f32out ? launch_typed<f16_t, float>(d, c, wf, x, y, s) : launch_typed<f16_t, f16_t>(d, c, wf, x, y, s);
    return f32out ? launch_typed<bf16_t, float>(d, c, wf, x, y, s) : launch_typed<bf16_t, bf16_t>(d, c, wf, x, y, s);
}

}  // namespace rtoss
