// Index arithmetic of the kernel-native sign layout, shared by the host repacker
// and the device kernels of this library.
//
// A tile covers 16 rows x 256 columns of every path.  Lane l = r + 16*q of a
// wavefront (r = row in the tile, q = 0..3) owns 2*K consecutive 32-bit words:
// word index c*K + k holds path k, row r, tile columns 128*c + 32*q .. +31, in
// canonical bit order (bit b = column +b, 1 means -1).  Tiles are stored
// row-tile major, so a wavefront that walks one row tile along the columns reads
// one contiguous run with one 8*K-byte load per lane per tile.
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

}  // namespace rb
