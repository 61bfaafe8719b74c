// Geometry of the activation tile the 3x3 matrix-core kernels keep in LDS.
#pragma once

namespace rtoss {

// One position of a stage: 32 channels x 2 bytes + 16 bytes of padding.  The padding makes the
// position pitch 80 bytes, which spreads the 16-byte operand reads of neighbouring positions
// over the LDS banks.
constexpr int kXPosBytes = 80;

// Output tile of (4*RT) x (4*CT) positions at stride S, made of RT x CT blocks of 4x4 positions
// (one block = the 16 columns of a matrix instruction).
template <int S, int RT, int CT> struct Geom {
    static constexpr int TH = 4 * RT, TW = 4 * CT;                      // output tile
    static constexpr int IH = (TH - 1) * S + 3, IW = (TW - 1) * S + 3;  // input tile with halo
    static constexpr int LW = ((IW + 3) / 8) * 8 + 4;                   // row pitch in positions, == 4 (mod 8), >= IW
    static constexpr int x_bytes = IH * LW * kXPosBytes;
    static constexpr int x_chunks = IH * IW * 4;                        // 16-byte chunks to fetch per stage
};

}  // namespace rtoss
