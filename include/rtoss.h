/*
 * rtoss.h -- C ABI of the MI355X (gfx950) hot path of R-TOSS pattern pruning.
 *
 * Three steps, each one or a few kernel launches on a caller-supplied HIP stream:
 *
 *   rtoss_select_patterns   per-kernel best pattern      (Section IV.C, Algorithm 2;
 *                                                          Section IV.D, Algorithm 3)
 *   rtoss_pack              prune + compact weight layout (Section II.B mask semantics;
 *                                                          Section IV.C, last sentence:
 *                                                          kernels laid out by pattern)
 *   rtoss_conv2d_pattern    convolution over the surviving weights only
 *                                                         (Section II.B cost model)
 *
 * plus the host-side dictionary generator rtoss_pattern_dict (Section IV.B, Eq. 1 and the
 * adjacency criterion) and the usage-based dictionary reduction of the same section
 * (rtoss_pattern_histogram on the device, rtoss_reduce_dict on the host).
 *
 * Conventions shared by every call
 *   - Pointers named *_dev are device (HBM) pointers, pointers named *_host are host
 *     pointers.  The library allocates no device memory and keeps no pointer after a call
 *     returns: every buffer is caller-owned.  Host arrays (the dictionary) are copied into
 *     the launch arguments before the call returns.
 *   - hip_stream is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *     validate their arguments on the host BEFORE touching the GPU, enqueue their kernels
 *     and return without synchronising.
 *   - Return value: RTOSS_OK or an error code; rtoss_last_error() gives a thread-local,
 *     statically stored message for the last failing call on this thread.  No exception
 *     crosses the boundary.
 *   - Tap numbering: a "group" is 9 contiguous weights; tap t is offset t in the group,
 *     i.e. row t/3, column t%3 of a 3x3 kernel.  A pattern is a uint16_t with bit t set
 *     iff tap t survives.  A dictionary is an array of P such masks that all have the
 *     same number k of set bits (one k per call: the paper's 2EP/3EP/4EP/5EP variants are
 *     separate dictionaries, Table 3), 1 <= P <= 255.
 *   - Determinism: identical inputs give bit-identical outputs (no atomics are used in any
 *     accumulation).
 *   - Activations are finite numbers.  (A pruned weight is an exact zero; zero times a
 *     non-finite activation is not defined by this interface.)
 */
#ifndef RTOSS_H
#define RTOSS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    RTOSS_OK = 0,
    RTOSS_EINVAL = 1,   /* NULL pointer, bad enum value, bad dictionary, misaligned pointer */
    RTOSS_ESHAPE = 2,   /* unsupported kernel size / stride / padding / extent */
    RTOSS_EDTYPE = 3,   /* unsupported dtype combination */
    RTOSS_ELAYOUT = 4,  /* unsupported activation layout */
    RTOSS_ENOSPACE = 5, /* a caller buffer is smaller than the size the library asked for */
    RTOSS_EHIP = 6      /* the HIP runtime reported an error (text in rtoss_last_error) */
} rtoss_status;

typedef enum { RTOSS_F32 = 0, RTOSS_F16 = 1, RTOSS_BF16 = 2 } rtoss_dtype;

typedef enum { RTOSS_NCHW = 0, RTOSS_NHWC = 1 } rtoss_layout;

/* Which k-subsets of the 9 taps enter the dictionary (Section IV.B: "drop all patterns
 * without adjacent non-zero weights").  The paper's figure of example patterns is not
 * reproducible from its text, so the reading is a parameter:
 *   ALL         every k-subset (Eq. 1 only);
 *   ANYPAIR4    at least one pair of edge-sharing live taps;
 *   CONNECTED4  the live taps form one edge-connected set (the default reading);
 *   CONNECTED8  connected when corner-sharing taps also count as neighbours.
 * A single tap (k = 1) passes every rule. */
typedef enum {
    RTOSS_RULE_ALL = 0,
    RTOSS_RULE_ANYPAIR4 = 1,
    RTOSS_RULE_CONNECTED4 = 2,
    RTOSS_RULE_CONNECTED8 = 3
} rtoss_rule;

/*
 * Section IV.B, Eq. 1 + first narrowing criterion.  Host only, no GPU needed.
 * Enumerates the k-subsets of taps {0..8} as ascending tuples in lexicographic order and
 * keeps those that pass `rule`; pattern index = rank among the kept ones.
 *   k      1..9
 *   masks  host array of `cap` entries, may be NULL when cap == 0 (count query)
 *   P      out: number of patterns in the dictionary (always the full count)
 * Returns RTOSS_EINVAL for a bad k / rule / NULL P, RTOSS_ENOSPACE when cap > 0 is smaller
 * than the count (the first cap masks are still written).
 */
rtoss_status rtoss_pattern_dict(int k, rtoss_rule rule, uint16_t* masks_host, int cap, int* P);

/*
 * Section IV.C (Algorithm 2: score every dictionary pattern on every kernel, keep the
 * best) on the flat view of Section IV.D (Algorithm 3: the weight tensor flattened
 * row-major and cut into groups of 9; for a [Co][Ci][3][3] tensor the groups are its
 * kernels, group g = co*Ci + ci).
 *
 *   w_dev       n_elems contiguous weights of type dt (device), aligned to its element size
 *   n_elems     >= 0; G = n_elems / 9 groups are scored, the n_elems % 9 tail is ignored
 *   masks_host  dictionary, P masks of equal popcount (host)
 *   idx_dev     out: G bytes (device); idx[g] = index of the pattern that maximises the
 *               retained energy  sum_{t live} w[9g+t]^2
 *
 * Arithmetic is fixed so that the result is reproducible bit for bit: each weight is
 * converted exactly to fp64, squares are summed in fp64 over the live taps in ascending
 * tap order starting from 0, patterns are scanned in ascending index with a strict
 * "greater than", so ties go to the lowest index, a NaN score never wins, and a group
 * whose every score is NaN gets index 0.
 * Several tensors may be scored by one call on their concatenation only if each has a
 * multiple of 9 elements (3x3 layers); a 1x1 tensor needs its own call because its tail
 * is per tensor.
 */
rtoss_status rtoss_select_patterns(const void* w_dev, rtoss_dtype dt, int64_t n_elems,
                                   const uint16_t* masks_host, int P,
                                   uint8_t* idx_dev, void* hip_stream);

/*
 * The same selection for several weight tensors of one dtype with one dictionary (all layers of a
 * model), in as few launches as possible: each tensor is selected exactly as by
 * rtoss_select_patterns (its own groups of 9, its own tail).
 *
 *   items_host  n_items entries {w_dev, n_elems, idx_dev} with the meaning and alignment of
 *               rtoss_select_patterns' arguments; the array is read before the call returns
 * Errors: as rtoss_select_patterns; RTOSS_EINVAL also for n_items < 0 or items_host NULL.
 */
typedef struct {
    const void* w_dev;
    int64_t n_elems;
    uint8_t* idx_dev;
} rtoss_select_item;
rtoss_status rtoss_select_patterns_batch(const rtoss_select_item* items_host, int n_items, rtoss_dtype dt,
                                         const uint16_t* masks_host, int P, void* hip_stream);

/*
 * Section IV.B, second narrowing criterion (keep the patterns that are used most when
 * the selection runs over random kernels), part 1: how often each pattern was selected.
 *     hist_dev[p] += #{ g < G : idx_dev[g] == p }      for p < P
 *
 *   idx_dev   G pattern indices from rtoss_select_patterns (device); values >= P are ignored
 *   hist_dev  P counters of type uint32 (device), 4-byte aligned.  The call ADDS to them, so
 *             that several tensors can be accumulated; the caller clears them before the
 *             first call.  Counts are integers: the result does not depend on the order in
 *             which the adds happen.
 * Errors: RTOSS_EINVAL (NULL, G < 0, P outside 1..255, misaligned hist_dev).
 */
rtoss_status rtoss_pattern_histogram(const uint8_t* idx_dev, int64_t G, int P,
                                     uint32_t* hist_dev, void* hip_stream);

/*
 * Section IV.B, second narrowing criterion, part 2.  Host only, no GPU needed.  Keeps the M
 * most used patterns of a dictionary: patterns are ranked by count, higher first, equal
 * counts by lower index; the M best are written to out_masks_host in their ORIGINAL
 * relative order, so that ties in a later selection over the reduced dictionary resolve
 * towards the same pattern as before.
 *
 *   masks_host      P masks (as for rtoss_select_patterns)
 *   hist_host       P counts (host copy of what rtoss_pattern_histogram accumulated)
 *   M               1..P
 *   out_masks_host  out: M masks
 *   kept_host       out, may be NULL: kept_host[i] = index in masks_host of out_masks_host[i]
 * How many random kernels to draw, and the number 21 the paper arrives at for its mixed
 * 2- and 3-entry dictionary, are not recoverable from the paper: M is the caller's choice.
 * Errors: RTOSS_EINVAL (NULL, bad dictionary, M outside 1..P).
 */
rtoss_status rtoss_reduce_dict(const uint16_t* masks_host, int P, const uint32_t* hist_host,
                               int M, uint16_t* out_masks_host, uint8_t* kept_host);

/* One convolution layer's weight tensor: [Co][Ci][ksize][ksize] contiguous, ksize 1 or 3,
 * k = number of survivors per group of 9 (the popcount of the dictionary's masks). */
typedef struct {
    int Co, Ci;
    int ksize; /* 1 or 3 */
    int k;     /* 1..9 */
    rtoss_dtype dt;
} rtoss_wdesc;

/*
 * Size in bytes of the packed blob rtoss_pack writes for this layer and dictionary, and
 * of the scratch workspace it needs (may be 0).  Host only.  The blob size depends on the
 * dictionary because the dictionary decides which compute layouts are legal (see below).
 */
rtoss_status rtoss_pack_size(const rtoss_wdesc* desc, const uint16_t* masks_host, int P,
                             size_t* packed_bytes, size_t* workspace_bytes);

/*
 * Prune and pack one layer (Section II.B: a mask keeps the weights it covers, the others
 * become zero; Section IV.D: the n_elems % 9 tail of a flattened 1x1 tensor is pruned;
 * Section IV.C, closing sentences: kernels are laid out by their pattern so that
 * inference touches only the survivors).
 *
 *   w_dev         the unpruned weights, Co*Ci*ksize*ksize elements of desc->dt (device)
 *   idx_dev       G = Co*Ci*ksize*ksize / 9 pattern indices from rtoss_select_patterns
 *   packed_dev    out: packed_bytes from rtoss_pack_size, 256-byte aligned (device).
 *                 The blob is position independent: it may be copied, saved and reloaded.
 *   workspace_dev scratch of workspace_bytes (may be NULL when that size is 0)
 *
 * Blob layout.  Section 0, always present and part of this interface (the tests decode it):
 *     [G][k]  surviving weights of each group in ascending tap order, type desc->dt
 *     [G]     pattern index of each group (uint8), starting at the next multiple of 256 B
 * Further sections (each starting at a multiple of 256 bytes) are private to the
 * convolution kernels: tiles of the pruned weights arranged as matrix-core operand
 * fragments, dense with explicit zeros or 2-of-4 compressed when every pattern of the
 * dictionary allows it.
 * Errors: RTOSS_EINVAL (NULL, bad dictionary, popcount != desc->k, misaligned blob),
 * RTOSS_ESHAPE (ksize not 1 or 3, non-positive extents), RTOSS_ENOSPACE.
 */
rtoss_status rtoss_pack(const rtoss_wdesc* desc, const void* w_dev, const uint8_t* idx_dev,
                        const uint16_t* masks_host, int P,
                        void* packed_dev, size_t packed_bytes,
                        void* workspace_dev, size_t workspace_bytes, void* hip_stream);

/*
 * rtoss_pack for several layers of one model that share a dictionary, in as few launches as
 * possible (layers whose private section has the same format and dtype are packed by one
 * launch).  Each item is packed exactly as by rtoss_pack; no workspace is needed.
 *
 *   items_host  n_items entries {desc, w_dev, idx_dev, packed_dev, packed_bytes} with the meaning
 *               of rtoss_pack's arguments; the array is read before the call returns
 * Errors: as rtoss_pack (the message names the item); nothing is launched if any item is invalid.
 */
typedef struct {
    rtoss_wdesc desc;
    const void* w_dev;
    const uint8_t* idx_dev;
    void* packed_dev;
    size_t packed_bytes;
} rtoss_pack_item;
rtoss_status rtoss_pack_batch(const rtoss_pack_item* items_host, int n_items,
                              const uint16_t* masks_host, int P, void* hip_stream);

/* One convolution call. */
typedef struct {
    int N, H, W;         /* batch, input height, input width */
    int stride;          /* 1 or 2 (1 only for ksize 1) */
    int pad;             /* must equal ksize / 2 */
    rtoss_layout layout; /* RTOSS_NHWC: x is [N][H][W][Ci], y is [N][Ho][Wo][Co];
                            RTOSS_NCHW: x is [N][Ci][H][W], y is [N][Co][Ho][Wo] */
    rtoss_dtype out_dt;  /* the weight dtype, or RTOSS_F32 */
    int fuse_relu;       /* non-zero: y = max(y, 0) */
} rtoss_cdesc;

/*
 * Convolution over the pruned weights (cross-correlation, zero padding, no bias, groups 1,
 * dilation 1), multiplying only surviving taps:
 *     y[n][oh][ow][co] = sum_ci sum_{t live in kernel (co,ci)}
 *                            w[co][ci][t] * x[n][oh*stride - pad + t/3][ow*stride - pad + t%3][ci]
 * with Ho = (H + 2*pad - ksize)/stride + 1 (same for Wo); for ksize 1 the weight matrix is
 * the pruned [Co][Ci] matrix of Section IV.D.
 *
 *   packed_dev  blob from rtoss_pack for the same desc and dictionary
 *   x_dev       activations of type desc->dt, 16-byte aligned; must not overlap y_dev
 *   y_dev       out: type cdesc->out_dt, 16-byte aligned
 * Products are accumulated in fp32 (inputs fp16/bf16/fp32 are multiplied exactly or in
 * fp32); the result is rounded once (nearest-even) when out_dt is a 16-bit type.
 * Layouts: the matrix-core kernels stream channels-last tensors (RTOSS_NHWC), which is the fast
 * path; RTOSS_NCHW tensors are served for every shape by the element-wise vector-ALU kernel
 * (same results, far slower: convert once instead where speed matters).
 * Errors: RTOSS_ESHAPE, RTOSS_EDTYPE, RTOSS_EINVAL (also for an unknown layout).
 */
rtoss_status rtoss_conv2d_pattern(const rtoss_wdesc* desc, const rtoss_cdesc* cdesc,
                                  const uint16_t* masks_host, int P,
                                  const void* packed_dev, const void* x_dev, void* y_dev,
                                  void* hip_stream);

/*
 * The same convolution with a fused output stage (the operations that follow a convolution in the
 * detector blocks whose inference time Section V reports: folded batch normalisation, activation,
 * shortcut connection):
 *     y = act(scale[co] * conv + bias[co]) + residual
 * evaluated in fp32 on the accumulator and rounded once on store.
 *
 *   scale_dev, bias_dev  Co floats each (device, 16-byte aligned), or NULL for 1 / 0
 *   act                  RTOSS_ACT_NONE, RTOSS_ACT_RELU (max(v, 0)) or RTOSS_ACT_SILU (v / (1 + exp(-v)))
 *   residual_dev         tensor of y's type and shape (device, 16-byte aligned), or NULL; may not
 *                        overlap y_dev
 *   y_ld, residual_ld    channels-last only: number of elements from one position's first channel
 *                        to the next position's, for y and for the residual; 0 means Co (a plain
 *                        tensor).  A larger value makes the tensor a channel slice of a wider
 *                        buffer: with y_dev = buffer + first_channel and y_ld = the buffer's channel
 *                        count, the convolution writes its Co channels of every position straight
 *                        into its place in a concatenation (the blocks of the detectors of Section V
 *                        concatenate branch outputs along channels), and other slices of the buffer
 *                        are left untouched.  Both must be multiples of 16 bytes and >= Co; the
 *                        slice's first element keeps the 16-byte alignment of y_dev / residual_dev.
 * cdesc->fuse_relu must be 0 (use act).  All other arguments and errors as rtoss_conv2d_pattern;
 * RTOSS_EINVAL also for a bad act, misaligned pointers or pitches, or fuse_relu != 0; RTOSS_ESHAPE
 * for a pitch below Co; RTOSS_ELAYOUT for a non-zero pitch with RTOSS_NCHW.
 */
typedef enum { RTOSS_ACT_NONE = 0, RTOSS_ACT_RELU = 1, RTOSS_ACT_SILU = 2 } rtoss_act;
typedef struct {
    const float* scale_dev;
    const float* bias_dev;
    rtoss_act act;
    const void* residual_dev;
    int y_ld;
    int residual_ld;
} rtoss_epilogue;
rtoss_status rtoss_conv2d_pattern_fused(const rtoss_wdesc* desc, const rtoss_cdesc* cdesc,
                                        const rtoss_epilogue* epilogue,
                                        const uint16_t* masks_host, int P,
                                        const void* packed_dev, const void* x_dev, void* y_dev,
                                        void* hip_stream);

/*
 * Layers whose kernels share their patterns in blocks (Section IV.A: the layers of a group take their
 * kernel patterns from the group's parent layer; Section IV.C, closing sentences: kernels with the same
 * pattern are processed together).  Where whole blocks of kernels -- 64 output channels x 8 consecutive
 * input channels, the granularity at which the dense matrix instruction shares its operands -- keep the same
 * taps, only those taps need a multiply at all: every multiply-add is then a non-zero one.
 *
 * rtoss_pack_coherent examines every block, records per (stage of 32 input channels, block of 64 output
 * channels) the number of dense steps it needs -- the largest number of distinct live taps among the stage's
 * four 8-channel runs: k when the patterns are shared, up to 9 when they are not -- and lays the weights out
 * for exactly those steps.  rtoss_conv2d_pattern_coherent computes the same convolution as
 * rtoss_conv2d_pattern from such a blob, for ANY index tensor; it is the faster call when the step counts
 * are small (below 5 on the layers that would otherwise take the 2-of-4 layout).
 *
 *   desc          3x3 layers of RTOSS_F16 / RTOSS_BF16 with Ci % 32 == 0, Ci <= 2048 and Co % 16 == 0
 *                 (RTOSS_ESHAPE / RTOSS_EDTYPE otherwise)
 *   steps_offset  out, may be NULL: byte offset in the blob of the detection result, one 64-byte record per
 *                 (stage, channel block), stage-major: uint32 steps; uint8 taps_per_run[4]; uint8 tap[4][9];
 *                 uint8 pad[20].  A caller that wants to choose between the two paths packs both ways or reads
 *                 these records back.
 *   epilogue      as for rtoss_conv2d_pattern_fused, or NULL for none (cdesc->fuse_relu is honoured then)
 * The blob's section 0 (survivors and indices) is the same as rtoss_pack's.  Channels-last tensors only
 * (RTOSS_ELAYOUT otherwise).  All other arguments and errors as rtoss_pack_size / rtoss_pack /
 * rtoss_conv2d_pattern_fused.
 */
rtoss_status rtoss_pack_size_coherent(const rtoss_wdesc* desc, const uint16_t* masks_host, int P,
                                      size_t* packed_bytes, size_t* steps_offset);
rtoss_status rtoss_pack_coherent(const rtoss_wdesc* desc, const void* w_dev, const uint8_t* idx_dev,
                                 const uint16_t* masks_host, int P,
                                 void* packed_dev, size_t packed_bytes, void* hip_stream);
rtoss_status rtoss_conv2d_pattern_coherent(const rtoss_wdesc* desc, const rtoss_cdesc* cdesc,
                                           const rtoss_epilogue* epilogue,
                                           const uint16_t* masks_host, int P,
                                           const void* packed_dev, const void* x_dev, void* y_dev,
                                           void* hip_stream);

/* Message for the last error on the calling thread ("" if none).  Static storage. */
const char* rtoss_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* RTOSS_H */
