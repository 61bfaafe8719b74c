// Host side of the C ABI: dictionary generation, argument validation, blob geometry and
// dispatch to the kernel launchers.  Every check happens before the first HIP call, so
// the error paths can be exercised on a machine without a GPU.
#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <vector>

#include "common.h"
#include "epilogue.h"

namespace rtoss {

static thread_local char g_err[512] = "";

rtoss_status fail(rtoss_status st, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return st;
}

rtoss_status check_hip(hipError_t e, const char* what)
{
    if (e == hipSuccess) return RTOSS_OK;
    return fail(RTOSS_EHIP, "%s: %s", what, hipGetErrorString(e));
}

rtoss_status current_device(DeviceInfo* out)
{
    constexpr int kSlots = 64;
    static std::atomic<int> cus_of[kSlots];  // 0 = not asked yet
    int dev = 0;
    if (rtoss_status st = check_hip(hipGetDevice(&dev), "hipGetDevice")) return st;
    int n = dev >= 0 && dev < kSlots ? cus_of[dev].load(std::memory_order_relaxed) : 0;
    if (n == 0) {
        if (rtoss_status st = check_hip(hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev), "compute unit count"))
            return st;
        if (n < 1) return fail(RTOSS_EHIP, "device %d reports %d compute units", dev, n);
        if (dev >= 0 && dev < kSlots) cus_of[dev].store(n, std::memory_order_relaxed);
    }
    out->device = dev;
    out->cus = n;
    return RTOSS_OK;
}

rtoss_status ensure_dynamic_lds(const void* kernel, size_t bytes, LaunchOnce& once, const char* what)
{
    int dev = 0;
    if (rtoss_status st = check_hip(hipGetDevice(&dev), "hipGetDevice")) return st;
    const bool tracked = dev >= 0 && dev < 64;
    if (tracked && (once.done.load(std::memory_order_acquire) >> dev & 1u)) return RTOSS_OK;
    if (rtoss_status st = check_hip(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes), what))
        return st;
    if (tracked) once.done.fetch_or((uint64_t)1 << dev, std::memory_order_release);
    return RTOSS_OK;
}

// ---------------------------------------------------------------------------------------
// Dictionary (Section IV.B): Eq. 1 candidates filtered by adjacency.
// ---------------------------------------------------------------------------------------
static unsigned neighbours_of(int t, bool eight)
{
    const int r = t / 3, c = t % 3;
    unsigned nb = 0;
    for (int dr = -1; dr <= 1; ++dr)
        for (int dc = -1; dc <= 1; ++dc) {
            if (!dr && !dc) continue;
            if (!eight && dr && dc) continue;
            const int rr = r + dr, cc = c + dc;
            if (rr >= 0 && rr < 3 && cc >= 0 && cc < 3) nb |= 1u << (rr * 3 + cc);
        }
    return nb;
}

static unsigned halo_of(unsigned set, bool eight)
{
    unsigned h = 0;
    for (int t = 0; t < 9; ++t)
        if (set >> t & 1u) h |= neighbours_of(t, eight);
    return h;
}

static bool one_component(unsigned m, bool eight)
{
    unsigned reach = m & (~m + 1u);  // lowest live tap
    for (;;) {
        const unsigned grown = reach | (halo_of(reach, eight) & m);
        if (grown == reach) break;
        reach = grown;
    }
    return reach == m;
}

static bool passes(unsigned m, rtoss_rule rule)
{
    switch (rule) {
    case RTOSS_RULE_ALL: return true;
    case RTOSS_RULE_ANYPAIR4: return __builtin_popcount(m) == 1 || (halo_of(m, false) & m) != 0;
    case RTOSS_RULE_CONNECTED4: return one_component(m, false);
    case RTOSS_RULE_CONNECTED8: return one_component(m, true);
    }
    return false;
}

static unsigned reverse9(unsigned m)
{
    unsigned r = 0;
    for (int t = 0; t < 9; ++t) r |= (m >> t & 1u) << (8 - t);
    return r;
}

// Validates a caller dictionary and copies it into launch-argument form.
static rtoss_status load_dict(const uint16_t* masks_host, int P, Dict* out)
{
    if (!masks_host) return fail(RTOSS_EINVAL, "dictionary pointer is NULL");
    if (P < 1 || P > kMaxPatterns) return fail(RTOSS_EINVAL, "dictionary size P=%d outside 1..%d", P, kMaxPatterns);
    std::memset(out, 0, sizeof *out);
    const int k = __builtin_popcount(masks_host[0]);
    for (int p = 0; p < P; ++p) {
        const unsigned m = masks_host[p];
        if (m == 0 || m > 0x1ffu) return fail(RTOSS_EINVAL, "pattern %d (0x%x) is not a non-empty 9-bit mask", p, m);
        if (__builtin_popcount(m) != k)
            return fail(RTOSS_EINVAL, "pattern %d keeps %d taps but pattern 0 keeps %d: one k per dictionary", p,
                        __builtin_popcount(m), k);
        out->mask[p] = (uint16_t)m;
    }
    out->P = P;
    out->k = k;
    return RTOSS_OK;
}

static rtoss_status check_wdesc(const rtoss_wdesc* d)
{
    if (!d) return fail(RTOSS_EINVAL, "weight descriptor is NULL");
    if (d->ksize != 1 && d->ksize != 3) return fail(RTOSS_ESHAPE, "ksize %d: only 1 and 3 are supported", d->ksize);
    if (d->Co < 1 || d->Ci < 1) return fail(RTOSS_ESHAPE, "Co=%d Ci=%d must be positive", d->Co, d->Ci);
    if ((int64_t)d->Co * d->Ci * d->ksize * d->ksize > (int64_t)1 << 40) return fail(RTOSS_ESHAPE, "weight tensor too large");
    if (d->dt != RTOSS_F32 && d->dt != RTOSS_F16 && d->dt != RTOSS_BF16) return fail(RTOSS_EDTYPE, "bad weight dtype %d", (int)d->dt);
    if (d->k < 1 || d->k > 9) return fail(RTOSS_EINVAL, "k=%d outside 1..9", d->k);
    return RTOSS_OK;
}

rtoss_status blob_geometry(const rtoss_wdesc* d, const Dict& dict, BlobGeometry* g, bool coherent)
{
    std::memset(g, 0, sizeof *g);
    g->n_elems = (int64_t)d->Co * d->Ci * d->ksize * d->ksize;
    g->G = g->n_elems / 9;
    g->live_off = 0;
    g->idx_off = align_up((size_t)g->G * d->k * elem_bytes(d->dt), 256);
    size_t end = align_up(g->idx_off + (size_t)g->G, 256);
    g->format = kFormatNone;
    g->mat_off = 0;
    g->mat_bytes = 0;
    if (coherent) {
        if (!gather3x3_shape_ok(*d))
            return fail(RTOSS_ESHAPE, "the coherent path takes 3x3 layers of a 16-bit type with Ci %% 32 == 0, Ci <= 2048, Co %% 16 == 0");
        g->format = kFormatGather3x3;
        g->mat_off = end;
        g->mat_bytes = gather3x3_section_bytes(*d);
        end = align_up(end + g->mat_bytes, 256);
    } else if (sparse3x3_shape_ok(*d) && sparse3x3_layout(dict) >= 0) {
        g->format = kFormatSparse24;
        g->mat_off = end;
        g->mat_bytes = sparse3x3_section_bytes(*d, sparse3x3_layout(dict));
        end = align_up(end + g->mat_bytes, 256);
    } else if (stem3x3_shape_ok(*d)) {
        g->format = kFormatStem;
        g->mat_off = end;
        g->mat_bytes = stem3x3_section_bytes(*d);
        end = align_up(end + g->mat_bytes, 256);
    } else if (dense3x3_shape_ok(*d)) {
        g->format = kFormatDense3x3;
        g->mat_off = end;
        g->mat_bytes = dense3x3_section_bytes(*d);
        end = align_up(end + g->mat_bytes, 256);
    } else if (stream1x1_shape_ok(*d)) {
        g->format = kFormatDenseStream;
        g->mat_off = end;
        g->mat_bytes = stream1x1_section_bytes(*d);
        end = align_up(end + g->mat_bytes, 256);
    } else if (dense1x1_shape_ok(*d)) {
        g->format = kFormatDense;
        g->mat_off = end;
        g->mat_bytes = dense1x1_section_bytes(*d);
        end = align_up(end + g->mat_bytes, 256);
    }
    g->total = std::max<size_t>(end, 256);
    return RTOSS_OK;
}

static bool misaligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) != 0; }

}  // namespace rtoss

using namespace rtoss;

extern "C" {

const char* rtoss_last_error(void) { return g_err; }

rtoss_status rtoss_pattern_dict(int k, rtoss_rule rule, uint16_t* masks_host, int cap, int* P)
{
    if (!P) return fail(RTOSS_EINVAL, "P is NULL");
    if (k < 1 || k > 9) return fail(RTOSS_EINVAL, "k=%d outside 1..9", k);
    if ((int)rule < 0 || (int)rule > 3) return fail(RTOSS_EINVAL, "unknown rule %d", (int)rule);
    if (cap < 0 || (cap > 0 && !masks_host)) return fail(RTOSS_EINVAL, "masks is NULL but cap=%d", cap);
    // Lexicographic order of ascending tap tuples == descending order of the bit-reversed mask.
    std::vector<unsigned> kept;
    for (unsigned m = 1; m < 512; ++m)
        if (__builtin_popcount(m) == k && passes(m, rule)) kept.push_back(m);
    std::sort(kept.begin(), kept.end(), [](unsigned a, unsigned b) { return reverse9(a) > reverse9(b); });
    *P = (int)kept.size();
    for (int i = 0; i < cap && i < (int)kept.size(); ++i) masks_host[i] = (uint16_t)kept[i];
    if (cap > 0 && cap < (int)kept.size()) return fail(RTOSS_ENOSPACE, "dictionary has %d patterns, cap is %d", *P, cap);
    return RTOSS_OK;
}

rtoss_status rtoss_select_patterns(const void* w_dev, rtoss_dtype dt, int64_t n_elems, const uint16_t* masks_host, int P,
                                   uint8_t* idx_dev, void* hip_stream)
{
    if (dt != RTOSS_F32 && dt != RTOSS_F16 && dt != RTOSS_BF16) return fail(RTOSS_EDTYPE, "bad dtype %d", (int)dt);
    if (n_elems < 0) return fail(RTOSS_EINVAL, "n_elems=%lld is negative", (long long)n_elems);
    Dict dict;
    if (rtoss_status st = load_dict(masks_host, P, &dict)) return st;
    const int64_t G = n_elems / 9;
    if (G == 0) return RTOSS_OK;
    if (!w_dev || !idx_dev) return fail(RTOSS_EINVAL, "w_dev or idx_dev is NULL");
    if (misaligned(w_dev, elem_bytes(dt))) return fail(RTOSS_EINVAL, "w_dev is not aligned to its element size");
    return launch_select(w_dev, dt, G, dict, idx_dev, (hipStream_t)hip_stream);
}

rtoss_status rtoss_select_patterns_batch(const rtoss_select_item* items_host, int n_items, rtoss_dtype dt,
                                         const uint16_t* masks_host, int P, void* hip_stream)
{
    if (dt != RTOSS_F32 && dt != RTOSS_F16 && dt != RTOSS_BF16) return fail(RTOSS_EDTYPE, "bad dtype %d", (int)dt);
    if (n_items < 0) return fail(RTOSS_EINVAL, "n_items=%d is negative", n_items);
    Dict dict;
    if (rtoss_status st = load_dict(masks_host, P, &dict)) return st;
    if (n_items == 0) return RTOSS_OK;
    if (!items_host) return fail(RTOSS_EINVAL, "items_host is NULL");
    for (int i = 0; i < n_items; ++i) {
        const rtoss_select_item& it = items_host[i];
        if (it.n_elems < 0) return fail(RTOSS_EINVAL, "item %d: n_elems=%lld is negative", i, (long long)it.n_elems);
        if (it.n_elems / 9 == 0) continue;
        if (!it.w_dev || !it.idx_dev) return fail(RTOSS_EINVAL, "item %d: w_dev or idx_dev is NULL", i);
        if (misaligned(it.w_dev, elem_bytes(dt))) return fail(RTOSS_EINVAL, "item %d: w_dev is not aligned to its element size", i);
    }
    return launch_select_batch(items_host, n_items, dt, dict, (hipStream_t)hip_stream);
}

rtoss_status rtoss_pattern_histogram(const uint8_t* idx_dev, int64_t G, int P, uint32_t* hist_dev, void* hip_stream)
{
    if (G < 0) return fail(RTOSS_EINVAL, "G=%lld is negative", (long long)G);
    if (P < 1 || P > kMaxPatterns) return fail(RTOSS_EINVAL, "P=%d outside 1..%d", P, kMaxPatterns);
    if (!hist_dev) return fail(RTOSS_EINVAL, "hist_dev is NULL");
    if (misaligned(hist_dev, 4)) return fail(RTOSS_EINVAL, "hist_dev is not 4-byte aligned");
    if (G == 0) return RTOSS_OK;
    if (!idx_dev) return fail(RTOSS_EINVAL, "idx_dev is NULL");
    return launch_histogram(idx_dev, G, P, hist_dev, (hipStream_t)hip_stream);
}

rtoss_status rtoss_reduce_dict(const uint16_t* masks_host, int P, const uint32_t* hist_host, int M, uint16_t* out_masks_host,
                               uint8_t* kept_host)
{
    Dict dict;
    if (rtoss_status st = load_dict(masks_host, P, &dict)) return st;
    if (!hist_host || !out_masks_host) return fail(RTOSS_EINVAL, "hist_host or out_masks_host is NULL");
    if (M < 1 || M > P) return fail(RTOSS_EINVAL, "M=%d outside 1..P=%d", M, P);
    // rank: count descending, index ascending on equal counts; then restore dictionary order
    int order[256];
    for (int p = 0; p < P; ++p) order[p] = p;
    std::stable_sort(order, order + P, [&](int a, int b) { return hist_host[a] > hist_host[b]; });
    std::sort(order, order + M);
    for (int i = 0; i < M; ++i) {
        out_masks_host[i] = dict.mask[order[i]];
        if (kept_host) kept_host[i] = (uint8_t)order[i];
    }
    return RTOSS_OK;
}

rtoss_status rtoss_pack_size(const rtoss_wdesc* desc, const uint16_t* masks_host, int P, size_t* packed_bytes,
                             size_t* workspace_bytes)
{
    if (rtoss_status st = check_wdesc(desc)) return st;
    if (!packed_bytes || !workspace_bytes) return fail(RTOSS_EINVAL, "size output pointer is NULL");
    Dict dict;
    if (rtoss_status st = load_dict(masks_host, P, &dict)) return st;
    if (dict.k != desc->k) return fail(RTOSS_EINVAL, "dictionary keeps %d taps, descriptor says k=%d", dict.k, desc->k);
    BlobGeometry g;
    if (rtoss_status st = blob_geometry(desc, dict, &g)) return st;
    *packed_bytes = g.total;
    *workspace_bytes = 0;
    return RTOSS_OK;
}

// Validation shared by rtoss_pack and rtoss_pack_batch; fills the geometry and the section pointers.
static rtoss_status check_pack(const rtoss_wdesc* desc, const Dict& dict, const void* w_dev, const uint8_t* idx_dev,
                               void* packed_dev, size_t packed_bytes, BlobGeometry* g, PackItem* item, bool coherent = false)
{
    if (rtoss_status st = check_wdesc(desc)) return st;
    if (dict.k != desc->k) return fail(RTOSS_EINVAL, "dictionary keeps %d taps, descriptor says k=%d", dict.k, desc->k);
    if (rtoss_status st = blob_geometry(desc, dict, g, coherent)) return st;
    if (!packed_dev) return fail(RTOSS_EINVAL, "packed_dev is NULL");
    if (packed_bytes < g->total)
        return fail(RTOSS_ENOSPACE, "packed buffer has %zu bytes, %zu needed", packed_bytes, g->total);
    if (misaligned(packed_dev, 256)) return fail(RTOSS_EINVAL, "packed_dev is not 256-byte aligned");
    if (g->G > 0 && (!w_dev || !idx_dev)) return fail(RTOSS_EINVAL, "w_dev or idx_dev is NULL");
    if (misaligned(w_dev, elem_bytes(desc->dt))) return fail(RTOSS_EINVAL, "w_dev is not aligned to its element size");
    char* blob = (char*)packed_dev;
    item->d = *desc;
    item->w = w_dev;
    item->idx = idx_dev;
    item->section = blob + g->mat_off;
    item->live = blob + g->live_off;
    item->live_idx = (uint8_t*)(blob + g->idx_off);
    return RTOSS_OK;
}

// one launch per layer: the fragment packers also write the public section in their first blocks
static rtoss_status pack_one(const PackItem& it, const BlobGeometry& g, const Dict& dict, hipStream_t s)
{
    if (g.format == kFormatSparse24) return launch_pack_sparse3x3(it.d, it.w, it.idx, dict, it.section, it.live, it.live_idx, s);
    if (g.format == kFormatDense3x3) return launch_pack_dense3x3(it.d, it.w, it.idx, dict, it.section, it.live, it.live_idx, s);
    if (g.format == kFormatDenseStream) return launch_pack_stream1x1(it.d, it.w, it.idx, dict, it.section, it.live, it.live_idx, s);
    if (g.format == kFormatDense) return launch_pack_dense1x1(it.d, it.w, it.idx, dict, it.section, it.live, it.live_idx, s);
    if (g.format == kFormatStem) return launch_pack_stem3x3(it.d, it.w, it.idx, dict, it.section, it.live, it.live_idx, s);
    return launch_pack_live(it.d, it.w, it.idx, dict, it.live, it.live_idx, g.G, s);
}

rtoss_status rtoss_pack(const rtoss_wdesc* desc, const void* w_dev, const uint8_t* idx_dev, const uint16_t* masks_host,
                        int P, void* packed_dev, size_t packed_bytes, void* workspace_dev, size_t workspace_bytes,
                        void* hip_stream)
{
    (void)workspace_dev;
    (void)workspace_bytes;
    if (rtoss_status st = check_wdesc(desc)) return st;
    Dict dict;
    if (rtoss_status st = load_dict(masks_host, P, &dict)) return st;
    BlobGeometry g;
    PackItem it;
    if (rtoss_status st = check_pack(desc, dict, w_dev, idx_dev, packed_dev, packed_bytes, &g, &it)) return st;
    return pack_one(it, g, dict, (hipStream_t)hip_stream);
}

rtoss_status rtoss_pack_batch(const rtoss_pack_item* items_host, int n_items, const uint16_t* masks_host, int P,
                              void* hip_stream)
{
    if (n_items < 0) return fail(RTOSS_EINVAL, "n_items=%d is negative", n_items);
    Dict dict;
    if (rtoss_status st = load_dict(masks_host, P, &dict)) return st;
    if (n_items == 0) return RTOSS_OK;
    if (!items_host) return fail(RTOSS_EINVAL, "items_host is NULL");
    std::vector<PackItem> items((size_t)n_items);
    std::vector<BlobGeometry> geo((size_t)n_items);
    for (int i = 0; i < n_items; ++i) {
        const rtoss_pack_item& in = items_host[i];
        if (rtoss_status st = check_pack(&in.desc, dict, in.w_dev, in.idx_dev, in.packed_dev, in.packed_bytes, &geo[i], &items[i])) {
            std::string msg = rtoss_last_error();
            return fail(st, "item %d: %s", i, msg.c_str());
        }
    }
    hipStream_t s = (hipStream_t)hip_stream;
    // layers of the two common formats go out in batched launches, per dtype; the rest one by one
    for (int fmt : {(int)kFormatSparse24, (int)kFormatDenseStream})
        for (int dt : {(int)RTOSS_F16, (int)RTOSS_BF16}) {
            std::vector<PackItem> group;
            for (int i = 0; i < n_items; ++i)
                if ((int)geo[i].format == fmt && (int)items[i].d.dt == dt) group.push_back(items[i]);
            if (group.empty()) continue;
            const rtoss_status st = fmt == kFormatSparse24 ? launch_pack_sparse3x3_batch(group.data(), (int)group.size(), dict, s)
                                                           : launch_pack_stream1x1_batch(group.data(), (int)group.size(), dict, s);
            if (st) return st;
        }
    for (int i = 0; i < n_items; ++i) {
        if (geo[i].format == kFormatSparse24 || geo[i].format == kFormatDenseStream) continue;
        if (rtoss_status st = pack_one(items[i], geo[i], dict, s)) return st;
    }
    return RTOSS_OK;
}

static rtoss_status conv_impl(const rtoss_wdesc* desc, const rtoss_cdesc* c, const rtoss_epilogue* e,
                              const uint16_t* masks_host, int P, const void* packed_dev, const void* x_dev, void* y_dev,
                              void* hip_stream, bool coherent = false)
{
    if (rtoss_status st = check_wdesc(desc)) return st;
    if (!c) return fail(RTOSS_EINVAL, "conv descriptor is NULL");
    Dict dict;
    if (rtoss_status st = load_dict(masks_host, P, &dict)) return st;
    if (dict.k != desc->k) return fail(RTOSS_EINVAL, "dictionary keeps %d taps, descriptor says k=%d", dict.k, desc->k);
    if (c->layout != RTOSS_NHWC && c->layout != RTOSS_NCHW) return fail(RTOSS_EINVAL, "unknown layout %d", (int)c->layout);
    if (c->stride != 1 && c->stride != 2) return fail(RTOSS_ESHAPE, "stride %d: only 1 and 2 are supported", c->stride);
    if (desc->ksize == 1 && c->stride != 1) return fail(RTOSS_ESHAPE, "1x1 convolution supports stride 1 only");
    if (c->pad != desc->ksize / 2) return fail(RTOSS_ESHAPE, "pad %d must equal ksize/2 = %d", c->pad, desc->ksize / 2);
    if (c->N < 1 || c->H < 1 || c->W < 1) return fail(RTOSS_ESHAPE, "N=%d H=%d W=%d must be positive", c->N, c->H, c->W);
    if (c->out_dt != desc->dt && c->out_dt != RTOSS_F32)
        return fail(RTOSS_EDTYPE, "out_dt must be the weight dtype or fp32");
    const int64_t Ho = (c->H + 2 * c->pad - desc->ksize) / c->stride + 1;
    const int64_t Wo = (c->W + 2 * c->pad - desc->ksize) / c->stride + 1;
    if (Ho < 1 || Wo < 1) return fail(RTOSS_ESHAPE, "empty output %lldx%lld", (long long)Ho, (long long)Wo);
    if ((int64_t)c->N * c->H * c->W * desc->Ci >= (int64_t)1 << 40 || (int64_t)c->N * Ho * Wo * desc->Co >= (int64_t)1 << 40)
        return fail(RTOSS_ESHAPE, "activation tensor too large");
    if (!packed_dev || !x_dev || !y_dev) return fail(RTOSS_EINVAL, "packed_dev, x_dev or y_dev is NULL");
    if (misaligned(packed_dev, 256)) return fail(RTOSS_EINVAL, "packed_dev is not 256-byte aligned");
    if (misaligned(x_dev, 16) || misaligned(y_dev, 16)) return fail(RTOSS_EINVAL, "x_dev and y_dev must be 16-byte aligned");
    // Output / residual position pitch (channels-last): Co, or wider when the tensor is a channel slice of a
    // larger buffer.  Runs of 16 bytes are stored at once, so the pitch keeps every position 16-byte aligned.
    int ldy = desc->Co, ldr = desc->Co;
    if (e) {
        if (e->y_ld < 0 || e->residual_ld < 0) return fail(RTOSS_EINVAL, "y_ld and residual_ld must not be negative");
        if ((e->y_ld || e->residual_ld) && c->layout != RTOSS_NHWC)
            return fail(RTOSS_ELAYOUT, "y_ld / residual_ld describe channels-last tensors; they must be 0 for NCHW");
        if (e->y_ld) ldy = e->y_ld;
        if (e->residual_ld) ldr = e->residual_ld;
        if (ldy < desc->Co || ldr < desc->Co)
            return fail(RTOSS_ESHAPE, "y_ld=%d / residual_ld=%d is smaller than Co=%d", e->y_ld, e->residual_ld, desc->Co);
        if ((size_t)ldy * elem_bytes(c->out_dt) % 16 || (size_t)ldr * elem_bytes(c->out_dt) % 16)
            return fail(RTOSS_EINVAL, "y_ld and residual_ld must be multiples of 16 bytes");
    }
    const int64_t positions = (int64_t)c->N * Ho * Wo;
    if (positions * std::max(ldy, ldr) >= (int64_t)1 << 40) return fail(RTOSS_ESHAPE, "activation tensor too large");
    // bytes from a tensor's first element to just past its last (a slice ends Co elements into its last position)
    const auto span = [&](int ld) { return ((size_t)(positions - 1) * ld + desc->Co) * elem_bytes(c->out_dt); };
    const size_t xb = (size_t)c->N * c->H * c->W * desc->Ci * elem_bytes(desc->dt);
    const size_t yb = span(ldy);
    const char *xa = (const char*)x_dev, *ya = (const char*)y_dev;
    if (xa < ya + yb && ya < xa + xb) return fail(RTOSS_EINVAL, "x and y overlap");
    ConvParams cp;
    static_cast<rtoss_cdesc&>(cp) = *c;
    cp.ep = Epilogue{nullptr, nullptr, nullptr, c->fuse_relu ? 1 : 0, ldy, ldr};
    if (e) {
        if (c->fuse_relu) return fail(RTOSS_EINVAL, "fuse_relu must be 0 when an epilogue is given (use its act)");
        if (e->act != RTOSS_ACT_NONE && e->act != RTOSS_ACT_RELU && e->act != RTOSS_ACT_SILU)
            return fail(RTOSS_EINVAL, "unknown activation %d", (int)e->act);
        if (misaligned(e->scale_dev, 16) || misaligned(e->bias_dev, 16) || misaligned(e->residual_dev, 16))
            return fail(RTOSS_EINVAL, "scale_dev, bias_dev and residual_dev must be 16-byte aligned");
        // (two channel slices of one wider buffer interleave without sharing an element: the overlap test
        // applies to plain tensors only)
        const char* ra = (const char*)e->residual_dev;
        if (ra && ldy == desc->Co && ldr == desc->Co && ra < ya + yb && ya < ra + yb)
            return fail(RTOSS_EINVAL, "residual and y overlap");
        cp.ep = Epilogue{e->scale_dev, e->bias_dev, e->residual_dev, (int)e->act, ldy, ldr};
    }
    BlobGeometry g;
    if (rtoss_status st = blob_geometry(desc, dict, &g, coherent)) return st;
    const char* blob = (const char*)packed_dev;
    if (coherent) {
        if (c->layout != RTOSS_NHWC) return fail(RTOSS_ELAYOUT, "the coherent path takes channels-last tensors");
        return launch_conv3x3_gather(*desc, cp, blob + g.mat_off, x_dev, y_dev, (hipStream_t)hip_stream);
    }
    if (c->layout == RTOSS_NCHW)  // the element-wise kernel reads section 0 and takes any strides
        return launch_conv_direct(*desc, cp, dict, blob + g.live_off, (const uint8_t*)(blob + g.idx_off), x_dev, y_dev,
                                  (hipStream_t)hip_stream);
    if (g.format == kFormatSparse24)
        return launch_conv3x3_sparse(*desc, cp, sparse3x3_layout(dict), blob + g.mat_off, x_dev, y_dev, (hipStream_t)hip_stream);
    if (g.format == kFormatStem)
        return launch_conv3x3_stem(*desc, cp, blob + g.mat_off, x_dev, y_dev, (hipStream_t)hip_stream);
    if (g.format == kFormatDense3x3)
        return launch_conv3x3_dense(*desc, cp, blob + g.mat_off, x_dev, y_dev, (hipStream_t)hip_stream);
    if (g.format == kFormatDenseStream)
        return launch_conv1x1_stream(*desc, cp, blob + g.mat_off, x_dev, y_dev, (hipStream_t)hip_stream);
    if (g.format == kFormatDense)
        return launch_conv1x1_mma(*desc, cp, blob + g.mat_off, x_dev, y_dev, (hipStream_t)hip_stream);
    return launch_conv_direct(*desc, cp, dict, blob + g.live_off, (const uint8_t*)(blob + g.idx_off), x_dev, y_dev,
                              (hipStream_t)hip_stream);
}


rtoss_status rtoss_pack_size_coherent(const rtoss_wdesc* desc, const uint16_t* masks_host, int P, size_t* packed_bytes,
                                      size_t* steps_offset)
{
    if (rtoss_status st = check_wdesc(desc)) return st;
    if (!packed_bytes) return fail(RTOSS_EINVAL, "size output pointer is NULL");
    Dict dict;
    if (rtoss_status st = load_dict(masks_host, P, &dict)) return st;
    if (dict.k != desc->k) return fail(RTOSS_EINVAL, "dictionary keeps %d taps, descriptor says k=%d", dict.k, desc->k);
    BlobGeometry g;
    if (rtoss_status st = blob_geometry(desc, dict, &g, true)) return st;
    *packed_bytes = g.total;
    if (steps_offset) *steps_offset = g.mat_off;
    return RTOSS_OK;
}

rtoss_status rtoss_pack_coherent(const rtoss_wdesc* desc, const void* w_dev, const uint8_t* idx_dev, const uint16_t* masks_host,
                                 int P, void* packed_dev, size_t packed_bytes, void* hip_stream)
{
    if (rtoss_status st = check_wdesc(desc)) return st;
    Dict dict;
    if (rtoss_status st = load_dict(masks_host, P, &dict)) return st;
    BlobGeometry g;
    PackItem it;
    if (rtoss_status st = check_pack(desc, dict, w_dev, idx_dev, packed_dev, packed_bytes, &g, &it, true)) return st;
    return launch_pack_gather3x3(it.d, it.w, it.idx, dict, it.section, it.live, it.live_idx, (hipStream_t)hip_stream);
}

rtoss_status rtoss_conv2d_pattern_coherent(const rtoss_wdesc* desc, const rtoss_cdesc* c, const rtoss_epilogue* epilogue,
                                           const uint16_t* masks_host, int P, const void* packed_dev, const void* x_dev,
                                           void* y_dev, void* hip_stream)
{
    return conv_impl(desc, c, epilogue, masks_host, P, packed_dev, x_dev, y_dev, hip_stream, true);
}

rtoss_status rtoss_conv2d_pattern(const rtoss_wdesc* desc, const rtoss_cdesc* c, const uint16_t* masks_host, int P,
                                  const void* packed_dev, const void* x_dev, void* y_dev, void* hip_stream)
{
    return conv_impl(desc, c, nullptr, masks_host, P, packed_dev, x_dev, y_dev, hip_stream);
}

rtoss_status rtoss_conv2d_pattern_fused(const rtoss_wdesc* desc, const rtoss_cdesc* c, const rtoss_epilogue* epilogue,
                                        const uint16_t* masks_host, int P, const void* packed_dev, const void* x_dev,
                                        void* y_dev, void* hip_stream)
{
    if (!epilogue) return fail(RTOSS_EINVAL, "epilogue is NULL");
    return conv_impl(desc, c, epilogue, masks_host, P, packed_dev, x_dev, y_dev, hip_stream);
}

}  // extern "C"
