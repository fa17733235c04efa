// Index arithmetic of the kernel-native sign layout, shared by the host repacker
// and the device kernels of this library.
//
// A tile covers 16 rows x 256 columns of every path.  Lane l = r + 16*q of a
// wavefront (r = row in the tile, q = 0..3) owns 2*K consecutive 32-bit words:
// word index c*K + k holds path k, row r, tile columns 128*c + 32*q .. +31.
// Inside a native word the 32 columns are bit-interleaved: native bit 4*e + s
// (e = 0..7, s = 0..3) is column 8*s + e (1 means -1).  With this order a shift
// by 3 - s and one mask turn a word into the s-th fp4 operand register of the
// matrix instruction, and contraction index == column, so that 16 consecutive
// input columns are 16 consecutive bytes of the 8-bit right operand.  Tiles are
// stored row-tile major, so a wavefront that walks one row tile along the
// columns reads one contiguous run with one 8*K-byte load per lane per tile.
#pragma once
#include <cstddef>
#include <cstdint>

#if defined(__HIPCC__)
#define RB_HD __host__ __device__
#else
#define RB_HD
#endif

namespace rb {

constexpr int TILE_ROWS = 16;
constexpr int TILE_COLS = 256;

RB_HD constexpr int row_tiles(int out) { return (out + TILE_ROWS - 1) / TILE_ROWS; }
RB_HD constexpr int col_tiles(int in) { return (in + TILE_COLS - 1) / TILE_COLS; }
RB_HD constexpr int tile_words(int K) { return 64 * 2 * K; }
// position of (lane, column half c, path k) inside a tile, in words
RB_HD constexpr int lane_word(int lane, int c, int k, int K) { return lane * 2 * K + c * K + k; }
// canonical word index (column / 32) that lane group q, half c of column tile ct holds
RB_HD constexpr int tile_word_column(int ct, int c, int q) { return ct * 8 + c * 4 + q; }

// native bit position of column offset b (0..31) inside a word, and back
RB_HD constexpr int native_bit(int b) { return 4 * (b & 7) + (b >> 3); }
RB_HD constexpr int column_of_native_bit(int p) { return 8 * (p & 3) + (p >> 2); }

RB_HD inline uint32_t to_native_word(uint32_t canonical)
{
    uint32_t w = 0;
    for (int b = 0; b < 32; ++b) w |= ((canonical >> b) & 1u) << native_bit(b);
    return w;
}
RB_HD inline uint32_t to_canonical_word(uint32_t native)
{
    uint32_t w = 0;
    for (int p = 0; p < 32; ++p) w |= ((native >> p) & 1u) << column_of_native_bit(p);
    return w;
}

}  // namespace rb
