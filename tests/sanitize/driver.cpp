// Driver for the address/undefined-behaviour sanitizer run of the two pieces of host code that
// index memory by hand: the oracle's C routines and the library's packing / native tiling.
// Built and run by tests/test_sanitizers.py with -fsanitize=address,undefined; every buffer is
// allocated at its exact size so that an access one element past either end is reported.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "rabit.h"

extern "C" {
int orc_pack(const int8_t *signs, int K, int out, int in, uint32_t *packed);
int orc_unpack(const uint32_t *packed, int K, int out, int in, int8_t *signs);
int orc_effective_weight(const int8_t *signs, const double *g, const double *h, int K, int out, int in, double *What);
int orc_matmul(const double *What, const double *X, int out, int in, int T, double *Y);
}

static uint64_t state = 0x9e3779b97f4a7c15ull;
static uint32_t next_u32()
{
    state ^= state << 13; state ^= state >> 7; state ^= state << 17;
    return (uint32_t)(state >> 32);
}

#define CHECK(cond)                                                              \
    do {                                                                         \
        if (!(cond)) { std::printf("FAILED %s line %d\n", #cond, __LINE__); return 1; } \
    } while (0)

static int one_shape(int K, int out, int in, int T)
{
    const size_t n = (size_t)K * out * in, words = n / 32;
    // exact-size heap blocks (vectors may over-allocate)
    int8_t *signs = (int8_t *)std::malloc(n), *back = (int8_t *)std::malloc(n);
    uint32_t *packed = (uint32_t *)std::malloc(words * 4), *packed2 = (uint32_t *)std::malloc(words * 4);
    uint32_t *canon = (uint32_t *)std::malloc(words * 4);
    for (size_t i = 0; i < n; ++i) signs[i] = (next_u32() & 1u) ? (int8_t)-1 : (int8_t)1;

    CHECK(orc_pack(signs, K, out, in, packed) == 0);
    CHECK(rb_pack(signs, K, out, in, packed2) == RB_OK);
    CHECK(std::memcmp(packed, packed2, words * 4) == 0);          // the two packers agree bit for bit
    CHECK(orc_unpack(packed, K, out, in, back) == 0);
    CHECK(std::memcmp(signs, back, n) == 0);
    CHECK(rb_unpack(packed2, K, out, in, back) == RB_OK);
    CHECK(std::memcmp(signs, back, n) == 0);

    const size_t nbytes = rb_native_bytes(K, out, in);
    CHECK(nbytes > 0 && nbytes % 4 == 0);
    void *native = std::malloc(nbytes);
    CHECK(rb_repack_native(packed2, K, out, in, native) == RB_OK);
    CHECK(rb_unpack_native(native, K, out, in, canon) == RB_OK);
    CHECK(std::memcmp(canon, packed2, words * 4) == 0);

    double *g = (double *)std::malloc(sizeof(double) * K * out), *h = (double *)std::malloc(sizeof(double) * K * in);
    double *What = (double *)std::malloc(sizeof(double) * out * in);
    double *X = (double *)std::malloc(sizeof(double) * T * in), *Y = (double *)std::malloc(sizeof(double) * T * out);
    for (int i = 0; i < K * out; ++i) g[i] = (double)(next_u32() % 1000) / 500.0 - 1.0;
    for (int i = 0; i < K * in; ++i) h[i] = (double)(next_u32() % 1000) / 500.0 - 1.0;
    for (int i = 0; i < T * in; ++i) X[i] = (double)(next_u32() % 1000) / 500.0 - 1.0;
    CHECK(orc_effective_weight(signs, g, h, K, out, in, What) == 0);
    CHECK(orc_matmul(What, X, out, in, T, Y) == 0);
    // one output by the definition of Section 4.1, with the sums written out
    const int t = T - 1, i = out - 1;
    double y = 0.0;
    for (int k = 0; k < K; ++k) {
        double s = 0.0;
        for (int j = 0; j < in; ++j) s += signs[((size_t)k * out + i) * in + j] * h[(size_t)k * in + j] * X[(size_t)t * in + j];
        y += g[(size_t)k * out + i] * s;
    }
    const double got = Y[(size_t)t * out + i];
    CHECK(got - y < 1e-9 && y - got < 1e-9);

    std::free(signs); std::free(back); std::free(packed); std::free(packed2); std::free(canon); std::free(native);
    std::free(g); std::free(h); std::free(What); std::free(X); std::free(Y);
    return 0;
}

int main()
{
    // one row / one word; ragged row tiles (out not a multiple of 16) and column tiles (in not a
    // multiple of 256); every K the format allows
    const int shapes[][4] = {{1, 1, 32, 1}, {2, 5, 32, 2}, {3, 17, 96, 3}, {2, 33, 288, 1}, {3, 16, 256, 2},
                             {2, 47, 544, 3}, {1, 130, 1056, 1}};
    for (const auto &s : shapes)
        if (one_shape(s[0], s[1], s[2], s[3]) != 0) {
            std::printf("shape K=%d out=%d in=%d T=%d\n", s[0], s[1], s[2], s[3]);
            return 1;
        }
    // argument checks must return before touching memory
    uint32_t w = 0; int8_t b = 1;
    if (rb_pack(nullptr, 1, 1, 32, &w) != RB_ERR_NULL || rb_pack(&b, 1, 1, 33, &w) != RB_ERR_SHAPE ||
        rb_pack(&b, RB_MAX_K + 1, 1, 32, &w) != RB_ERR_SHAPE || rb_native_bytes(1, 1, 31) != 0) {
        std::printf("FAILED argument checks\n");
        return 1;
    }
    std::printf("sanitizer driver: all shapes passed\n");
    return 0;
}
