// Geometry of the activation tile the 3x3 matrix-core kernels keep in LDS.
#pragma once

namespace rtoss {

// One position of a stage: 32 channels x 2 bytes (or 16 x 4).  Stride 1 packs positions at a 64-byte pitch;
// with the row pitch below, the 16-byte operand reads of a 4x4 block of positions then spread over all LDS
// banks.  At stride 2 the same reads would hit every bank twice (measured: 64 instead of 32 cycles per read
// with four waves), so there a position carries 16 bytes of padding: 80-byte pitch.
template <int S> constexpr int kXPosBytesFor = S == 1 ? 64 : 80;

// Output tile of (4*RT) x (4*CT) positions at stride S, made of RT x CT blocks of 4x4 positions
// (one block = the 16 columns of a matrix instruction).
template <int S, int RT, int CT> struct Geom {
    static constexpr int TH = 4 * RT, TW = 4 * CT;                      // output tile
    static constexpr int IH = (TH - 1) * S + 3, IW = (TW - 1) * S + 3;  // input tile with halo
    static constexpr int LW = ((IW + 3) / 8) * 8 + 4;                   // row pitch in positions, == 4 (mod 8), >= IW
    static constexpr int kPos = kXPosBytesFor<S>;                       // position pitch in bytes
    static constexpr int kChunks = kPos / 16;                           // 16-byte chunks per position, padding included
    static constexpr int x_bytes = IH * LW * kPos;
    static constexpr int x_chunks = IH * IW * 4;                        // 16-byte chunks to fetch per stage
};

}  // namespace rtoss
