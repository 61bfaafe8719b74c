// Layout of the 2-of-4 compressed weight fragments that the packer writes and the 3x3 kernels on the
// sparse matrix instruction stream (conv3x3_sparse.hip, conv3x3_rows.hip).
#pragma once
#include "common.h"

namespace rtoss {

// Packed weight fragments: per (stage of 32 input channels, tile of 16 output channels)
//   5 operand fragments of 64 lanes x 16 bytes: corner step 0/1, edge step 0/1, centre
//   then 2 index words per lane: [corner][lane], [edge][lane]; low half = step 0, high = step 1
// (which output channel a row of a tile is: tile_row_channel)
constexpr int kFragBytes = 1024;
constexpr int kTileBytes = 5 * kFragBytes + 2 * 64 * 4;  // 5632
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
inline size_t fragment_bytes(const rtoss_wdesc& d) { return (size_t)(d.Ci / 32) * padded_m_tiles(d.Co) * kTileBytes; }
inline size_t zero_block_bytes(const rtoss_wdesc& d) { return align_up((size_t)2 * d.Ci + 16, 256); }

}  // namespace rtoss
