/*
 * CPU oracle for the residual-binary linear layer.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain definition the GPU library is checked against.
 * It shares no code, header, table or helper with the HIP sources, and only
 * the tests, the smoke check and the benchmark's CPU-baseline leg may call it.
 *
 * Everything is fp64 and written as the paper states it:
 *   - Section 4.1 ("Binary Building Blocks"): (W_hat)_ij = g_i * B_ij * h_j,
 *     B in {-1,+1}^{d_out x d_in}, g per output channel, h per input channel.
 *   - Eq. (stacked binary weight): W_hat^(k) = sum_i g_i (.) B_i (.) h_i.
 *   - Alg. 2, layer output: Y = W_hat^(k) X  (a dense product).
 *   - Appendix "Weight Packing": 32 columns per 32-bit word, +1 -> bit 0,
 *     -1 -> bit 1.  The paper does not fix the bit order inside a word; the
 *     reading taken here is least-significant bit = lowest column.
 *
 * OpenMP only spreads independent output rows over the host cores; there is
 * no blocking, fusion or re-association beyond the definition.
 */
#include <stddef.h>
#include <stdint.h>

/* Weight Packing: bit b of word w of row i of path k is 1 iff B_k[i][32w+b] == -1. */
int orc_pack(const int8_t *signs, int K, int out, int in, uint32_t *packed)
{
    if (!signs || !packed || K < 1 || out < 1 || in < 32 || in % 32 != 0)
        return -1;
    const int W32 = in / 32;
    for (int k = 0; k < K; ++k)
        for (int i = 0; i < out; ++i)
            for (int w = 0; w < W32; ++w) {
                uint32_t word = 0;
                for (int b = 0; b < 32; ++b) {
                    int8_t s = signs[((size_t)k * out + i) * in + 32 * w + b];
                    if (s != 1 && s != -1)
                        return -2;
                    if (s == -1)
                        word |= (uint32_t)1 << b;
                }
                packed[((size_t)k * out + i) * W32 + w] = word;
            }
    return 0;
}

/* Inverse of orc_pack. */
int orc_unpack(const uint32_t *packed, int K, int out, int in, int8_t *signs)
{
    if (!signs || !packed || K < 1 || out < 1 || in < 32 || in % 32 != 0)
        return -1;
    const int W32 = in / 32;
    for (int k = 0; k < K; ++k)
        for (int i = 0; i < out; ++i)
            for (int j = 0; j < in; ++j) {
                uint32_t word = packed[((size_t)k * out + i) * W32 + j / 32];
                signs[((size_t)k * out + i) * in + j] = ((word >> (j % 32)) & 1u) ? -1 : 1;
            }
    return 0;
}

/*
 * Eq. (stacked binary weight): What[i][j] = sum_k g_k[i] * B_k[i][j] * h_k[j].
 * signs int8 [K][out][in], g fp64 [K][out], h fp64 [K][in], What fp64 [out][in].
 */
int orc_effective_weight(const int8_t *signs, const double *g, const double *h,
                         int K, int out, int in, double *What)
{
    if (!signs || !g || !h || !What || K < 1 || out < 1 || in < 1)
        return -1;
#pragma omp parallel for schedule(static)
    for (int i = 0; i < out; ++i)
        for (int j = 0; j < in; ++j) {
            double w = 0.0;
            for (int k = 0; k < K; ++k)
                w += g[(size_t)k * out + i] * (double)signs[((size_t)k * out + i) * in + j] *
                     h[(size_t)k * in + j];
            What[(size_t)i * in + j] = w;
        }
    return 0;
}

/*
 * Alg. 2, "compute layer output": Y = What X, for T input vectors stored
 * token-major: X fp64 [T][in], Y fp64 [T][out], Y[t][i] = sum_j What[i][j] X[t][j].
 */
int orc_matmul(const double *What, const double *X, int out, int in, int T, double *Y)
{
    if (!What || !X || !Y || out < 1 || in < 1 || T < 1)
        return -1;
#pragma omp parallel for schedule(static)
    for (int i = 0; i < out; ++i)
        for (int t = 0; t < T; ++t) {
            double acc = 0.0;
            for (int j = 0; j < in; ++j)
                acc += What[(size_t)i * in + j] * X[(size_t)t * in + j];
            Y[(size_t)t * out + i] = acc;
        }
    return 0;
}

/* Number of threads the parallel loops above use (for reporting). */
#ifdef _OPENMP
#include <omp.h>
int orc_threads(void) { return omp_get_max_threads(); }
#else
int orc_threads(void) { return 1; }
#endif
