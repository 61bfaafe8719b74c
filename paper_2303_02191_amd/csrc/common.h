// Internal declarations shared by the host API and the kernel launchers.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

#include "rtoss.h"

namespace rtoss {

struct ConvParams;  // rtoss_cdesc + the fused output stage (epilogue.h)

constexpr int kMaxPatterns = 255;

// A dictionary travels to every kernel by value in the launch arguments, so the host
// array can be released as soon as the call returns and no device copy is needed.
struct Dict {
    uint16_t mask[256];
    int P;
    int k;
};

// Decoded dictionary for the convolution kernels: tap[p][j] = j-th live tap of pattern p
// in ascending order (unused entries 0).
struct TapTable {
    uint8_t tap[256][9];
};

inline int elem_bytes(rtoss_dtype dt) { return dt == RTOSS_F32 ? 4 : 2; }
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ----- packed blob geometry (host side; the kernels receive section pointers) -----
enum MatrixFormat {
    kFormatNone = 0,     // only the live list (section 0): direct kernels
    kFormatDense = 1,    // 1x1: zero-filled matrix-core fragments
    kFormatSparse24 = 2, // 3x3: 2-of-4 compressed fragments + indices
    kFormatStem = 3,     // 3x3 with <= 3 input channels: one zero-filled fragment per 16 output channels
    kFormatDenseStream = 4,  // 1x1 with Ci = 32 * 2^n <= 1024: zero-filled fragments in the streaming kernel's order
    kFormatDense3x3 = 5,     // 3x3 whose dictionary has no 2-of-4 shape: zero-filled fragments, one per tap
    kFormatGather3x3 = 6     // 3x3, on request (rtoss_pack_coherent): per-block tap lists on the dense instruction
};

struct BlobGeometry {
    int64_t G;          // number of groups of 9
    int64_t n_elems;    // Co*Ci*ksize*ksize
    size_t live_off;    // [G][k] values
    size_t idx_off;     // [G] bytes
    MatrixFormat format;
    size_t mat_off;     // matrix-core section (0 if none)
    size_t mat_bytes;
    size_t total;
};

// Filled by host code in api.cpp.
rtoss_status blob_geometry(const rtoss_wdesc* d, const Dict& dict, BlobGeometry* out, bool coherent = false);

// ----- error plumbing -----
rtoss_status fail(rtoss_status st, const char* fmt, ...);
rtoss_status check_hip(hipError_t e, const char* what);

// ----- per-device launch state (api.hip) -----
// The current device's ordinal and its number of compute units (queried once per device).
struct DeviceInfo {
    int device;
    int cus;
};
rtoss_status current_device(DeviceInfo* out);
// Raises a kernel's dynamic-LDS limit to `bytes` on the current device, once per (kernel instantiation,
// device): `done` is the instantiation's own word, bit d = done on device d.  Safe to call from several
// threads (the attribute call is idempotent; the word only saves repeating it).
struct LaunchOnce {
    std::atomic<uint64_t> done{0};
};
rtoss_status ensure_dynamic_lds(const void* kernel, size_t bytes, LaunchOnce& once, const char* what);

// ----- launchers (one per kernel family; defined next to the kernels) -----
rtoss_status launch_select(const void* w, rtoss_dtype dt, int64_t G, const Dict& dict, uint8_t* idx, hipStream_t s);

constexpr int kSelectBatchMax = 64;  // tensors per batched selection launch
rtoss_status launch_select_batch(const rtoss_select_item* items, int n, rtoss_dtype dt, const Dict& dict, hipStream_t s);

// counts of each pattern index (select.hip)
rtoss_status launch_histogram(const uint8_t* idx, int64_t G, int P, uint32_t* hist, hipStream_t s);

rtoss_status launch_pack_live(const rtoss_wdesc& d, const void* w, const uint8_t* idx, const Dict& dict,
                              void* live_values, uint8_t* live_idx, int64_t G, hipStream_t s);

rtoss_status launch_conv_direct(const rtoss_wdesc& d, const ConvParams& c, const Dict& dict, const void* live_values,
                                const uint8_t* live_idx, const void* x, void* y, hipStream_t s);

// Several layers packed by one launch (layers of one format and dtype; the table travels in the launch arguments).
struct PackItem {
    rtoss_wdesc d;
    const void* w;
    const uint8_t* idx;
    void* section;      // private section of the blob
    void* live;         // public section: values
    uint8_t* live_idx;  // public section: indices
};
constexpr int kPackBatchMax = 24;
// block -> (entry, block within the entry) for the batched kernels: first_block[t] <= block < first_block[t+1]
template <typename Batch> __device__ __forceinline__ int batch_entry(const Batch& b, int block)
{
    // binary search: the table sits in the kernel arguments, and every probe is a dependent scalar load
    int lo = 0, hi = b.n - 1;  // the entry is in [lo, hi]
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (block >= b.first_block[mid]) lo = mid;
        else hi = mid - 1;
    }
    return lo;
}
rtoss_status launch_pack_sparse3x3_batch(const PackItem* items, int n, const Dict& dict, hipStream_t s);
rtoss_status launch_pack_stream1x1_batch(const PackItem* items, int n, const Dict& dict, hipStream_t s);

// 3x3 convolution on the sparse matrix instruction (conv3x3_sparse.hip)
// which tap layout (sparse_frag.h) fits every pattern of the dictionary, cheapest first; -1: none
int sparse3x3_layout(const Dict& dict);
bool sparse3x3_shape_ok(const rtoss_wdesc& d);
size_t sparse3x3_section_bytes(const rtoss_wdesc& d, int layout);
rtoss_status launch_pack_sparse3x3(const rtoss_wdesc& d, const void* w, const uint8_t* idx, const Dict& dict,
                                   void* section, void* live_values, uint8_t* live_idx, hipStream_t s);
rtoss_status launch_conv3x3_sparse(const rtoss_wdesc& d, const ConvParams& c, int layout, const void* section, const void* x,
                                   void* y, hipStream_t s);

// ... large stride-1 layers: pipelined kernel over strips of output rows (conv3x3_rows.hip); same packed section
rtoss_status launch_conv3x3_rows(const rtoss_wdesc& d, const ConvParams& c, const void* section, const void* x, void* y,
                                 hipStream_t s);

// 3x3 convolution with live taps gathered onto the dense matrix instruction, for block-shared patterns
// (conv3x3_gather.hip); its own blob format, chosen by the caller (rtoss_pack_coherent)
bool gather3x3_shape_ok(const rtoss_wdesc& d);
size_t gather3x3_header_bytes(const rtoss_wdesc& d);
size_t gather3x3_section_bytes(const rtoss_wdesc& d);
rtoss_status launch_pack_gather3x3(const rtoss_wdesc& d, const void* w, const uint8_t* idx, const Dict& dict, void* section,
                                   void* live_values, uint8_t* live_idx, hipStream_t s);
rtoss_status launch_conv3x3_gather(const rtoss_wdesc& d, const ConvParams& c, const void* section, const void* x, void* y,
                                   hipStream_t s);

// 3x3 convolution in dense mode on the matrix cores (conv3x3_dense.hip)
bool dense3x3_shape_ok(const rtoss_wdesc& d);
size_t dense3x3_section_bytes(const rtoss_wdesc& d);
rtoss_status launch_pack_dense3x3(const rtoss_wdesc& d, const void* w, const uint8_t* idx, const Dict& dict, void* section,
                                  void* live_values, uint8_t* live_idx, hipStream_t s);
rtoss_status launch_conv3x3_dense(const rtoss_wdesc& d, const ConvParams& c, const void* section, const void* x, void* y,
                                  hipStream_t s);

// 1x1 convolution on the dense matrix instruction (conv1x1_mma.hip)
bool dense1x1_shape_ok(const rtoss_wdesc& d);
size_t dense1x1_section_bytes(const rtoss_wdesc& d);
rtoss_status launch_pack_dense1x1(const rtoss_wdesc& d, const void* w, const uint8_t* idx, const Dict& dict, void* section,
                                  void* live_values, uint8_t* live_idx, hipStream_t s);
rtoss_status launch_conv1x1_mma(const rtoss_wdesc& d, const ConvParams& c, const void* section, const void* x, void* y,
                                hipStream_t s);

// 1x1 convolution, streaming kernel with register-resident weights (conv1x1_stream.hip)
bool stream1x1_shape_ok(const rtoss_wdesc& d);
size_t stream1x1_section_bytes(const rtoss_wdesc& d);
rtoss_status launch_pack_stream1x1(const rtoss_wdesc& d, const void* w, const uint8_t* idx, const Dict& dict, void* section,
                                   void* live_values, uint8_t* live_idx, hipStream_t s);
rtoss_status launch_conv1x1_stream(const rtoss_wdesc& d, const ConvParams& c, const void* section, const void* x, void* y,
                                   hipStream_t s);

// 3x3 convolution with <= 3 input channels (conv3x3_stem.hip)
bool stem3x3_shape_ok(const rtoss_wdesc& d);
size_t stem3x3_section_bytes(const rtoss_wdesc& d);
rtoss_status launch_pack_stem3x3(const rtoss_wdesc& d, const void* w, const uint8_t* idx, const Dict& dict, void* section,
                                 void* live_values, uint8_t* live_idx, hipStream_t s);
rtoss_status launch_conv3x3_stem(const rtoss_wdesc& d, const ConvParams& c, const void* section, const void* x, void* y,
                                 hipStream_t s);

}  // namespace rtoss
