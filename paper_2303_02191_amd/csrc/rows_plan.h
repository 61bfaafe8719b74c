// Row-strip tiling shared by the pipelined 3x3 kernels (conv3x3_rows.hip, conv3x3_gather.hip): how the rows of
// the 16-column strips are cut into tiles and dealt to persistent workgroups.
#pragma once

#include "common.h"

namespace rtoss {

constexpr int kTall = 5, kShort = 4;  // output rows per wave of the two tile classes
constexpr int kRowsTM = 8;             // channel tiles per workgroup (128 channels)
constexpr int kLW = 18;               // LDS row pitch of the activation tile in positions: 16 columns + halo
constexpr int kPosBytes = 64;         // one position of a stage: 32 channels x 2 bytes

// How the rows of the strips are cut into tiles, and how the tiles are dealt to the workgroups.
// A strip is 16 output columns of one image.  Strips [0, sa) are cut into a5 tall tiles followed by a4
// short ones, the other strips into b5 tall and b4 short.  A list entry is (tile, channel block) with the
// channel block fastest; each class has its own list, cut into 8 contiguous ranges, one per XCD, so that
// the channel blocks of a tile, and neighbouring tiles, meet in one L2.
struct RowPlan {
    int col_strips, co_blocks, strips;
    int sa, a5, a4, b5, b4;
    int tall_total, tall_per_xcd, short_total, short_per_xcd;
};

struct TileCoord {
    int n_img, mt0, oh0, ow0;
};

__device__ __forceinline__ TileCoord decode_entry(const RowPlan& p, bool tall, int e)
{
    const int na = tall ? p.a5 : p.a4, nb = tall ? p.b5 : p.b4;
    const int first_a = na * p.co_blocks * p.sa;  // entries of the strips cut the first way
    int strip, r, row0;
    if (e < first_a) {
        strip = e / (na * p.co_blocks);
        r = e - strip * (na * p.co_blocks);
        row0 = tall ? 0 : p.a5 * (4 * kTall);
    } else {
        const int e2 = e - first_a;
        const int s2 = e2 / (nb * p.co_blocks);
        strip = p.sa + s2;
        r = e2 - s2 * (nb * p.co_blocks);
        row0 = tall ? 0 : p.b5 * (4 * kTall);
    }
    const int tile = r / p.co_blocks, cblk = r - tile * p.co_blocks;
    TileCoord t;
    t.n_img = strip / p.col_strips;
    t.ow0 = (strip - t.n_img * p.col_strips) * 16;
    t.oh0 = row0 + tile * (tall ? 4 * kTall : 4 * kShort);
    t.mt0 = cblk * kRowsTM;
    return t;
}


// The cut of a launch shape into tall and short tiles with the smallest busiest-workgroup cost, for `slots`
// workgroups per XCD and `stages` stages of 32 input channels per tile; results are remembered per shape.
RowPlan plan_rows(int N, int H, int W, int co_blocks, int stages, int slots);
// One workgroup per compute unit, fewer when the tile lists are shorter: sets *slots (workgroups per XCD; the grid
// is 8 * slots) and returns the plan for it.
RowPlan plan_rows_for_device(int N, int H, int W, int co_blocks, int stages, int cus, int* slots);

}  // namespace rtoss
