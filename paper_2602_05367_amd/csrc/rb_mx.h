// Matrix-core path of the residual-binary layer: plan structures shared by the
// host planner and the device kernels, and the layout of the expanded input.
//
// Section 4.1: y = sum_k g_k (.) (B_k (h_k (.) x)).  The inner product B_k u_k
// with u_k = h_k (.) x is a contraction of a +-1 matrix with a vector.  On
// gfx950 the vector ALUs cannot apply one sign per packed bit as fast as HBM
// delivers the bits, so the signs are expanded to fp4 (E2M1) +-1 operands with
// two vector instructions per eight weights and contracted by
// v_mfma_scale_f32_16x16x128_f8f6f4 against u_k held as a sum of four bf8
// (E5M2) terms: u = t1 + t2/8 + t3/64 + t4/512, each term the bf8 rounding of
// the remaining residual times 8.  The four terms, for both paths (and for up
// to two tokens), sit in different columns of the 16-column right operand, so
// the expansion costs no additional matrix instructions.
#pragma once
#include <cstddef>
#include <cstdint>

#include "rabit.h"

namespace rb {
namespace mx {

constexpr int CWAVES = 8;          // wavefronts that stream weights and issue MFMAs
constexpr int EWAVES = 4;          // wavefronts that finish rows and talk to other CUs
constexpr int THREADS = (CWAVES + EWAVES) * 64;
constexpr int RING_D = 12;         // sign tiles in flight per compute wavefront (1 KB each)
constexpr int NB = 4;              // expanded-input operands in flight per compute wavefront (tiles)
constexpr int MAXSLOT = 8;         // (op, row tile) pairs one CU finishes per stage
constexpr int MAX_CONS = 3;        // ops that read one op's output inside a fused stack
constexpr int MAX_T = 2;           // tokens per call on this path
static_assert(RING_D > NB && 5 * NB - 4 <= 63, "the in-order wait counts on this");

constexpr int LDS_RING_BYTES = CWAVES * RING_D * 1024;
constexpr int LDS_PART_BYTES = 2 * MAXSLOT * 2048;
constexpr int LDS_MISC_BYTES = 256 + CWAVES * 256;   // counters + per-wavefront dummy-load target
constexpr int LDS_BYTES = LDS_RING_BYTES + LDS_PART_BYTES + LDS_MISC_BYTES;

// Expanded input ("right operand") of one op: for every 128-column block cb
// there are 16 operand columns of 128 bytes: column 8*(token&1) + 4*path + term.
// Inside a column, the byte that multiplies input column j of the block sits
// where the MFMA pairs it with the fp4 sign taken from bit (j % 32) of the
// canonical word j / 32 (see operand_byte).
constexpr int UP_BLOCK_BYTES = 16 * 128;

// byte offset inside a 128-byte operand column for input column jj (0..127)
__host__ __device__ inline int operand_byte(int jj)
{
    const int q = jj >> 5, o = jj & 31;        // lane group that owns the word, bit in word
    const int s = o & 3, e = o >> 2;           // fp4 register s, nibble e  (bit = 4*e + s)
    const int k = 32 * q + 8 * s + e;          // contraction index of that nibble
    // the 8-bit operand keeps k in [16*q', 16*q'+16) and [64+16*q', 64+16*q'+16) in lane group q'
    return k < 64 ? (k >> 4) * 32 + (k & 15) : ((k - 64) >> 4) * 32 + 16 + ((k - 64) & 15);
}

struct Op {
    const uint32_t *bits;     // native sign tiles
    const uint16_t *g;        // fp16 [K][out]
    const uint16_t *h;        // fp16 [K][in]
    const uint16_t *x;        // fp16 [T][in]  input buffer (read by the expansion kernel only)
    uint16_t *y;              // fp16 [T][out] output buffer
    uint8_t *up;              // expanded input of this op: [pairs][CB][16][128] bytes
    int out, in;
    int RT, CT;               // row tiles (16 rows), column tiles (256 columns)
    int n_cons;               // ops that read y inside this call
    int cons[MAX_CONS];
    int expand_x;             // 1: x comes from outside the fused ops and must be expanded first
    int pad_;
    float sc[2];              // power-of-two input scale per path (max |h| * sc <= 1/2)
    float inv_sc[2];
};

struct Stage {
    int op0, nops;            // ops [op0, op0 + nops) are independent of each other
    int wait_before;          // 1: an op of this stage reads what an earlier stage wrote
    int signal_after;         // 1: a later stage reads what this stage writes
};

struct Header {
    int n_ops, n_stages, T, n_groups;
    uint32_t epoch0;          // barrier epoch of the first signalling stage of this launch
    uint32_t pad_[3];
};

// workspace: [Header][Op x n_ops][Stage x n_stages][flags: n_groups x u32][error u32][zero page 128 B][up arrays]
struct Layout {
    size_t ops, stages, flags, error, zero, up, total;
};

__host__ __device__ inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

__host__ __device__ inline size_t up_bytes(int in, int T)
{
    const int CB = (in + 255) / 256 * 2;
    return (size_t)((T + 1) / 2) * CB * UP_BLOCK_BYTES;
}

}  // namespace mx
}  // namespace rb
