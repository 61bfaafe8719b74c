// Direct pattern-sparse convolution on the vector ALUs (fp32 accumulate).
//
// This is the path for layers the matrix cores do not fit: fp32 tensors, very small
// channel counts, any shape the fragment layouts do not cover, and NCHW activations (the
// matrix-core kernels stream channels-last tensors).  It multiplies only
// the k surviving taps of every kernel (Section II.B: zero weights are skipped).
//
// Mapping: a workgroup owns an 8x8 tile of output positions (one position per lane) and a
// block of output channels; each of its 4 wavefronts owns kCoPerWave of those channels, so
// the weight and its tap offset are wave-uniform and every lane reads the activation tile
// in LDS at "own position + uniform tap offset", which is conflict free for stride 1.
// Per chunk of input channels the workgroup stages, into LDS, (a) the activation tile with
// its halo as fp32, channel-major, and (b) for every (output channel, input channel) pair
// of the block its k live weights as fp32 and the k LDS offsets of their taps.  The inner
// loop then touches LDS only: one broadcast read of the weights, one of the offsets and k
// activation reads per pair, with no dependent global loads in flight.
#include "common.h"
#include "dtypes.h"
#include "epilogue.h"

namespace rtoss {

constexpr int kTile = 8;        // output tile is kTile x kTile positions
constexpr int kCoPerWave = 4;   // accumulators per lane
constexpr int kWaves = 4;
constexpr int kCoPerBlock = kCoPerWave * kWaves;
constexpr int kChunk = 16;      // input channels staged per round
constexpr int kPairs = kCoPerBlock * kChunk;

// Element strides of the activation tensors: the kernel reads and writes one element at a time, so it serves
// both layouts of the interface (channels-last, and NCHW) and channel slices of wider channels-last buffers.
struct TensorStrides {
    int64_t n, h, w, c;
};
struct DirectStrides {
    TensorStrides x, y, r;  // input, output, residual
};

template <int KS, int S> struct Halo {
    static constexpr int side = (kTile - 1) * S + KS;
    static constexpr int count = side * side;
    static constexpr int padded = count | 1;  // odd row length: channel-major writes spread over banks
};

// KK = entries per kernel known at compile time (2, 3, 4), or 0: read k at run time.
// For 1x1 layers every pair carries exactly one weight (zero when pruned) at offset 0.
template <typename T, typename TO, int KS, int S, int KK>
__global__ __launch_bounds__(256) void conv_direct_kernel(const T* __restrict__ x, TO* __restrict__ y,
                                                          const T* __restrict__ live, const uint8_t* __restrict__ lidx,
                                                          Dict dict, int N, int H, int W, int Ci, int Co, int Ho, int Wo,
                                                          int tiles_w, Epilogue ep, int64_t G, DirectStrides st)
{
    using HL = Halo<KS, S>;
    constexpr int WS = KS == 1 ? 1 : (KK ? KK : 9);  // weights (and offsets) stored per pair
    __shared__ float xs[kChunk * HL::padded];
    __shared__ __align__(16) float wl[kPairs * WS];
    __shared__ __align__(16) int16_t ol[kPairs * WS];
    __shared__ int16_t tapoff[KS == 3 ? 256 * 9 : 1];  // LDS offset of the j-th live tap of pattern p
    __shared__ uint16_t masks[256];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tile = blockIdx.x;
    const int th = tile / tiles_w, tw = tile % tiles_w;
    const int n = blockIdx.z;
    const int co_block = blockIdx.y * kCoPerBlock;
    const int k = KS == 1 ? 1 : (KK ? KK : dict.k);

    masks[tid] = dict.mask[tid];
    if (KS == 3) {
        const unsigned m = dict.mask[tid];
        int j = 0;
        for (int t = 0; t < 9; ++t)
            if ((m >> t) & 1u) tapoff[tid * 9 + j++] = (int16_t)((t / 3) * HL::side + (t % 3));
        for (; j < 9; ++j) tapoff[tid * 9 + j] = 0;
    }

    const int oh0 = th * kTile, ow0 = tw * kTile;
    const int ih0 = oh0 * S - (KS / 2), iw0 = ow0 * S - (KS / 2);
    const int r = lane / kTile, c = lane % kTile;
    const int base = (r * S) * HL::side + c * S;

    float acc[kCoPerWave];
#pragma unroll
    for (int i = 0; i < kCoPerWave; ++i) acc[i] = 0.f;

    for (int ci0 = 0; ci0 < Ci; ci0 += kChunk) {
        const int nch = Ci - ci0 < kChunk ? Ci - ci0 : kChunk;
        __syncthreads();  // previous chunk fully consumed (also orders the table writes above)
        // (consecutive lanes read consecutive addresses: channels when they are contiguous, else positions)
        const bool channels_fastest = st.x.c == 1;
        for (int e = tid; e < HL::count * kChunk; e += 256) {
            const int ch = channels_fastest ? e % kChunk : e / HL::count;
            const int pos = channels_fastest ? e / kChunk : e % HL::count;
            const int ih = ih0 + pos / HL::side, iw = iw0 + pos % HL::side;
            float v = 0.f;
            if (ch < nch && ih >= 0 && ih < H && iw >= 0 && iw < W)
                v = to_f32(x[n * st.x.n + ih * st.x.h + iw * st.x.w + (ci0 + ch) * st.x.c]);
            xs[ch * HL::padded + pos] = v;
        }
        // Weights of this chunk.  Pairs outside the layer (channel tails) get weight 0 at
        // offset 0, so the inner loop needs no bounds test.
        for (int e = tid; e < kPairs; e += 256) {
            const int ch = e % kChunk, col = e / kChunk;
            const int co = co_block + col;
            const bool inside = co < Co && ch < nch;
            if (KS == 3) {
                const int64_t g = (int64_t)co * Ci + ci0 + ch;
                const int p = inside ? lidx[g] : 0;
                for (int j = 0; j < k; ++j) {
                    wl[e * WS + j] = inside ? to_f32(live[g * k + j]) : 0.f;
                    ol[e * WS + j] = inside ? tapoff[p * 9 + j] : (int16_t)0;
                }
            } else {
                // 1x1: the 9-groups run along the flattened [Co][Ci] matrix and may
                // straddle rows; element f belongs to group f/9 at tap f%9.
                float v = 0.f;
                if (inside) {
                    const int64_t f = (int64_t)co * Ci + ci0 + ch;
                    const int64_t g = f / 9;
                    const int t = (int)(f - g * 9);
                    if (g < G) {
                        const unsigned m = masks[lidx[g]];
                        if ((m >> t) & 1u) v = to_f32(live[g * dict.k + __builtin_popcount(m & ((1u << t) - 1u))]);
                    }
                }
                wl[e] = v;
                ol[e] = 0;
            }
        }
        __syncthreads();

        const float* xb = xs + base;
        for (int ch = 0; ch < kChunk; ++ch) {
            const float* xc = xb + ch * HL::padded;
#pragma unroll
            for (int i = 0; i < kCoPerWave; ++i) {
                const int e = ((wave * kCoPerWave + i) * kChunk + ch) * WS;
                if (KS == 1) {
                    acc[i] += wl[e] * xc[0];
                } else if (KK) {
#pragma unroll
                    for (int j = 0; j < KK; ++j) acc[i] += wl[e + j] * xc[ol[e + j]];
                } else {
                    for (int j = 0; j < k; ++j) acc[i] += wl[e + j] * xc[ol[e + j]];
                }
            }
        }
    }

    const int oh = oh0 + r, ow = ow0 + c;
    if (oh < Ho && ow < Wo) {
        TO* yp = y + n * st.y.n + oh * st.y.h + ow * st.y.w;
        const TO* rp = (const TO*)ep.residual + n * st.r.n + oh * st.r.h + ow * st.r.w;
#pragma unroll
        for (int i = 0; i < kCoPerWave; ++i) {
            const int co = co_block + wave * kCoPerWave + i;
            if (co < Co) {
                float v = acc[i];
                if (ep.scale) v *= ep.scale[co];
                if (ep.bias) v += ep.bias[co];
                v = epi_act(v, ep.act);
                if (ep.residual) v += to_f32(rp[co * st.r.c]);
                store_from_f32<TO>(yp + co * st.y.c, v);
            }
        }
    }
}

template <typename T, typename TO>
static rtoss_status launch_typed(const rtoss_wdesc& d, const ConvParams& c, const Dict& dict, const void* live,
                                 const uint8_t* lidx, const void* x, void* y, hipStream_t s)
{
    const int Ho = (c.H + 2 * c.pad - d.ksize) / c.stride + 1;
    const int Wo = (c.W + 2 * c.pad - d.ksize) / c.stride + 1;
    const int tiles_h = (Ho + kTile - 1) / kTile, tiles_w = (Wo + kTile - 1) / kTile;
    const int64_t G = (int64_t)d.Co * d.Ci * d.ksize * d.ksize / 9;
    if (c.N > 65535 || (d.Co + kCoPerBlock - 1) / kCoPerBlock > 65535)
        return fail(RTOSS_ESHAPE, "conv: batch or channel count too large for the direct kernel");
    dim3 grid((unsigned)(tiles_h * tiles_w), (unsigned)((d.Co + kCoPerBlock - 1) / kCoPerBlock), (unsigned)c.N);
    dim3 block(256);
    DirectStrides st;
    if (c.layout == RTOSS_NCHW) {
        st.x = TensorStrides{(int64_t)d.Ci * c.H * c.W, c.W, 1, (int64_t)c.H * c.W};
        st.y = TensorStrides{(int64_t)d.Co * Ho * Wo, Wo, 1, (int64_t)Ho * Wo};
        st.r = st.y;
    } else {
        st.x = TensorStrides{(int64_t)c.H * c.W * d.Ci, (int64_t)c.W * d.Ci, d.Ci, 1};
        st.y = TensorStrides{(int64_t)Ho * Wo * c.ep.ldy, (int64_t)Wo * c.ep.ldy, c.ep.ldy, 1};
        st.r = TensorStrides{(int64_t)Ho * Wo * c.ep.ldr, (int64_t)Wo * c.ep.ldr, c.ep.ldr, 1};
    }
#define RTOSS_LAUNCH(KS, S, KK)                                                                                  \
    conv_direct_kernel<T, TO, KS, S, KK><<<grid, block, 0, s>>>((const T*)x, (TO*)y, (const T*)live, lidx, dict, c.N, \
                                                                c.H, c.W, d.Ci, d.Co, Ho, Wo, tiles_w, c.ep, G, st)
#define RTOSS_LAUNCH3(S)                  \
    switch (dict.k) {                     \
    case 2: RTOSS_LAUNCH(3, S, 2); break; \
    case 3: RTOSS_LAUNCH(3, S, 3); break; \
    case 4: RTOSS_LAUNCH(3, S, 4); break; \
    default: RTOSS_LAUNCH(3, S, 0); break; \
    }
    if (d.ksize == 3 && c.stride == 1) { RTOSS_LAUNCH3(1) }
    else if (d.ksize == 3 && c.stride == 2) { RTOSS_LAUNCH3(2) }
    else if (d.ksize == 1 && c.stride == 1) RTOSS_LAUNCH(1, 1, 0);
    else return fail(RTOSS_ESHAPE, "conv: unsupported ksize/stride %d/%d", d.ksize, c.stride);
#undef RTOSS_LAUNCH3
#undef RTOSS_LAUNCH
    return check_hip(hipGetLastError(), "conv launch");
}

rtoss_status launch_conv_direct(const rtoss_wdesc& d, const ConvParams& c, const Dict& dict, const void* live_values,
                                const uint8_t* live_idx, const void* x, void* y, hipStream_t s)
{
    const bool f32out = c.out_dt == RTOSS_F32;
    switch (d.dt) {
    case RTOSS_F32: return launch_typed<float, float>(d, c, dict, live_values, live_idx, x, y, s);
    case RTOSS_F16:
        return f32out ? launch_typed<f16_t, float>(d, c, dict, live_values, live_idx, x, y, s)
                      : launch_typed<f16_t, f16_t>(d, c, dict, live_values, live_idx, x, y, s);
    case RTOSS_BF16:
        return f32out ? launch_typed<bf16_t, float>(d, c, dict, live_values, live_idx, x, y, s)
                      : launch_typed<bf16_t, bf16_t>(d, c, dict, live_values, live_idx, x, y, s);
    }
    return fail(RTOSS_EDTYPE, "conv: bad dtype");
}

}  // namespace rtoss
