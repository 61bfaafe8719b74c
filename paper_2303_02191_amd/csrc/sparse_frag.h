// Layout of the 2-of-4 compressed weight fragments that the packer writes and the 3x3 kernels on the
// sparse matrix instruction stream (conv3x3_sparse.hip, conv3x3_rows.hip).
#pragma once
#include "common.h"

namespace rtoss {

// How the 9 taps of a kernel are laid onto the matrix instructions: `groups` sets of up to 4 taps, each a
// 2-of-4 group of the sparse instruction (legal for a dictionary when no pattern has more than 2 live taps in
// any set; a set of 3 leaves its fourth slot empty), and optionally the centre tap as a dense K-slot.  Per
// 32 input channels a layout costs 2 sparse steps per group + 1 dense step for the centre, against 9 dense
// steps.  An exhaustive search over all partitions of the taps gives, for the edge-connected dictionaries:
//   2 and 3 entries: 5 steps (two groups of 4 + the centre: layout 0, corners / edge midpoints);
//   4 entries:       6 steps (three groups of 3, no tap left over: layout 1; the T shapes have 3 edge
//                    midpoints, so layout 0 does not fit them);
//   5 and more:      no partition is cheaper than the 9 dense steps.
struct TapLayout {
    int groups;     // sparse groups
    int centre;     // 1: tap 4 is a dense step of its own
    int tap[3][4];  // taps of each group's 4 slots, -1 = empty slot
};
constexpr int kNumLayouts = 2;
constexpr TapLayout kLayouts[kNumLayouts] = {
    {2, 1, {{0, 2, 6, 8}, {1, 3, 5, 7}, {-1, -1, -1, -1}}},
    {3, 0, {{0, 4, 8, -1}, {1, 5, 6, -1}, {2, 3, 7, -1}}},
};
// Packed weight fragments: per (stage of 32 input channels, tile of 16 output channels)
//   operand fragments of 64 lanes x 16 bytes: [group][step 0/1] ..., then the centre's if the layout has one
//   then one index word per lane and group: [group][lane]; low half = step 0, high = step 1
// (which output channel a row of a tile is: tile_row_channel)
constexpr int kFragBytes = 1024;
constexpr int layout_fragments(const TapLayout& l) { return 2 * l.groups + l.centre; }
constexpr int layout_tile_bytes(const TapLayout& l) { return layout_fragments(l) * kFragBytes + l.groups * 64 * 4; }
constexpr int kTileBytes = layout_tile_bytes(kLayouts[0]);  // 5632: layout 0, the only one the pipelined kernel takes
// 16-bit outputs without a fused output stage are stored straight from the accumulators (measured faster
// than the transposition through LDS once a lane's values are 32 contiguous bytes: tile_row_channel)
constexpr bool kDirectEpilogue = true;

// Output channel held by row r of channel tile mt.  Within a group of 4 tiles (64 channels) the rows
// are dealt so that the accumulator values one lane holds after the multiplication -- rows
// 4q .. 4q+3 of each of the 4 tiles -- are the 16 consecutive channels 64*(mt/4) + 16q .. +15:
// the epilogues store runs of 16 channels without exchanging data between lanes.
__device__ __forceinline__ int tile_row_channel(int mt, int r)
{
    return 64 * (mt >> 2) + 16 * (r >> 2) + 4 * (mt & 3) + (r & 3);
}
// first of the 4 consecutive channels that quarter q of a lane holds of tile mm (counted from the
// first channel of mm's group of 4 tiles when mm < 4; mm may run over several groups)
__device__ __forceinline__ int tile_quarter_offset(int mm, int q)
{
    return 64 * (mm >> 2) + 16 * q + 4 * (mm & 3);
}

// Channel tiles per stage in the packed section: padded so that every block of 8 tiles is complete.
inline int padded_m_tiles(int Co) { return ((Co + 15) / 16 + 7) / 8 * 8; }
// The section is [fragments][block of zeros]; the zeros feed the copy lanes that fill padding.
inline size_t fragment_bytes(const rtoss_wdesc& d, int layout = 0)
{
    return (size_t)(d.Ci / 32) * padded_m_tiles(d.Co) * layout_tile_bytes(kLayouts[layout]);
}
inline size_t zero_block_bytes(const rtoss_wdesc& d) { return align_up((size_t)2 * d.Ci + 16, 256); }

}  // namespace rtoss
