// Host-side packing: canonical sign words and the kernel-native tiling.
// Appendix "Weight Packing": 32 columns -> one 32-bit word, +1 -> 0, -1 -> 1.
#include "rabit.h"
#include "rb_layout.h"

#include <cstring>

extern "C" int rb_pack(const int8_t *signs, int K, int out, int in, uint32_t *packed)
{
    if (!signs || !packed) return RB_ERR_NULL;
    if (K < 1 || K > RB_MAX_K || out < 1 || in < 32 || in % 32 != 0) return RB_ERR_SHAPE;
    const size_t words_per_row = (size_t)in / 32;
    const size_t rows = (size_t)K * out;
    for (size_t row = 0; row < rows; ++row) {
        const int8_t *s = signs + row * in;
        uint32_t *dst = packed + row * words_per_row;
        for (size_t w = 0; w < words_per_row; ++w) {
            uint32_t word = 0;
            for (int b = 0; b < 32; ++b) {
                const int8_t v = s[32 * w + b];
                if (v == -1) word |= 1u << b;
                else if (v != 1) return RB_ERR_VALUE;
            }
            dst[w] = word;
        }
    }
    return RB_OK;
}

extern "C" int rb_unpack(const uint32_t *packed, int K, int out, int in, int8_t *signs)
{
    if (!signs || !packed) return RB_ERR_NULL;
    if (K < 1 || K > RB_MAX_K || out < 1 || in < 32 || in % 32 != 0) return RB_ERR_SHAPE;
    const size_t words_per_row = (size_t)in / 32;
    const size_t rows = (size_t)K * out;
    for (size_t row = 0; row < rows; ++row)
        for (size_t w = 0; w < words_per_row; ++w) {
            const uint32_t word = packed[row * words_per_row + w];
            for (int b = 0; b < 32; ++b)
                signs[row * in + 32 * w + b] = (word >> b) & 1u ? (int8_t)-1 : (int8_t)1;
        }
    return RB_OK;
}

extern "C" size_t rb_native_bytes(int K, int out, int in)
{
    if (K < 1 || K > RB_MAX_K || out < 1 || in < 32 || in % 32 != 0) return 0;
    return (size_t)rb::row_tiles(out) * rb::col_tiles(in) * rb::tile_words(K) * sizeof(uint32_t);
}

extern "C" int rb_repack_native(const uint32_t *packed, int K, int out, int in, void *native_host)
{
    if (!packed || !native_host) return RB_ERR_NULL;
    if (K < 1 || K > RB_MAX_K || out < 1 || in < 32 || in % 32 != 0) return RB_ERR_SHAPE;
    uint32_t *dst = static_cast<uint32_t *>(native_host);
    const int RT = rb::row_tiles(out), CT = rb::col_tiles(in), W32 = in / 32;
    for (int rt = 0; rt < RT; ++rt)
        for (int ct = 0; ct < CT; ++ct) {
            uint32_t *tile = dst + ((size_t)rt * CT + ct) * rb::tile_words(K);
            for (int lane = 0; lane < 64; ++lane) {
                const int row = rt * rb::TILE_ROWS + lane % 16, q = lane / 16;
                for (int c = 0; c < 2; ++c)
                    for (int k = 0; k < K; ++k) {
                        const int w = rb::tile_word_column(ct, c, q);
                        uint32_t v = 0;                         // padding: +1 everywhere
                        if (row < out && w < W32) v = rb::to_native_word(packed[((size_t)k * out + row) * W32 + w]);
                        tile[rb::lane_word(lane, c, k, K)] = v;
                    }
            }
        }
    return RB_OK;
}

extern "C" int rb_unpack_native(const void *native_host, int K, int out, int in, uint32_t *packed)
{
    if (!packed || !native_host) return RB_ERR_NULL;
    if (K < 1 || K > RB_MAX_K || out < 1 || in < 32 || in % 32 != 0) return RB_ERR_SHAPE;
    const uint32_t *src = static_cast<const uint32_t *>(native_host);
    const int CT = rb::col_tiles(in), W32 = in / 32;
    for (int k = 0; k < K; ++k)
        for (int row = 0; row < out; ++row)
            for (int w = 0; w < W32; ++w) {
                const int rt = row / rb::TILE_ROWS, r = row % rb::TILE_ROWS;
                const int ct = w / 8, c = (w % 8) / 4, q = w % 4;
                const uint32_t *tile = src + ((size_t)rt * CT + ct) * rb::tile_words(K);
                packed[((size_t)k * out + row) * W32 + w] = rb::to_canonical_word(tile[rb::lane_word(r + 16 * q, c, k, K)]);
            }
    return RB_OK;
}

extern "C" int rb_version(void) { return 100; }
