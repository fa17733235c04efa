// Matrix-core path of the residual-binary layer: plan structures shared by the
// host planner and the device kernels, and the layout of the expanded input.
//
// Section 4.1: y = sum_k g_k (.) (B_k (h_k (.) x)).  The inner product B_k u_k
// with u_k = h_k (.) x is a contraction of a +-1 matrix with a vector.  On
// gfx950 the vector ALUs cannot apply one sign per packed bit as fast as HBM
// delivers the bits, so the signs are expanded to fp4 (E2M1) +-1 operands with
// seven vector instructions per 32 weights and contracted by
// v_mfma_scale_f32_16x16x128_f8f6f4 against u_k held as a sum of four bf8
// (E5M2) terms: u = t0 + t1/8 + t2/64 + t3/512, each term the bf8 rounding of
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
constexpr int RING_D = 10;         // sign tiles in flight per compute wavefront (1 KB each)
constexpr int NB = 4;              // expanded-input operands in flight per compute wavefront (tiles)
constexpr int MAXSLOT = 8;         // (op, row tile) pairs one CU finishes per stage
constexpr int MAX_CONS = 3;        // ops that read one op's output inside a fused stack
constexpr int MAX_T = 2;           // tokens per call on this path
constexpr int MAX_OPS = 320;       // ops per launch (their per-wavefront records live in LDS)
constexpr size_t MAX_EXPAND = 1024;
static_assert(RING_D > NB && 5 * NB - 4 <= 63, "the in-order wait counts on this");

// LDS map of the stack kernel
constexpr int LDS_RING_BYTES = CWAVES * RING_D * 1024;
// partial sums: [parity][slot][compute wavefront][path][token][row] fp32
constexpr int LDS_PART_SLOT_BYTES = CWAVES * 2 * 2 * 16 * 4;
constexpr int LDS_PART_BYTES = 2 * MAXSLOT * LDS_PART_SLOT_BYTES;
constexpr int LDS_REC_BYTES = CWAVES * MAX_OPS * 8;      // WaveRec per (wavefront, op)
constexpr int LDS_INFO_BYTES = MAX_OPS * 32;             // OpInfo per op
constexpr int LDS_STAGE_BYTES = 2 * MAX_CONS * 2 * 2 * 4 * 16;   // per finishing wavefront: bytes of expanded outputs
constexpr int LDS_MISC_BYTES = 256 + CWAVES * 256 + EWAVES * LDS_STAGE_BYTES;   // + per-wavefront dummy-load target
constexpr int LDS_RING_OFF = 0;
constexpr int LDS_PART_OFF = LDS_RING_OFF + LDS_RING_BYTES;
constexpr int LDS_REC_OFF = LDS_PART_OFF + LDS_PART_BYTES;
constexpr int LDS_INFO_OFF = LDS_REC_OFF + LDS_REC_BYTES;
constexpr int LDS_MISC_OFF = LDS_INFO_OFF + LDS_INFO_BYTES;
constexpr int LDS_BYTES = LDS_MISC_OFF + LDS_MISC_BYTES;
static_assert(LDS_BYTES <= 160 * 1024, "LDS of one compute unit");

// Expanded input ("right operand") of one op: for every 128-column block cb
// there are 16 operand columns of 128 bytes: column 8*(token&1) + 4*path + term.
// Inside a column, the byte that multiplies input column j of the block sits
// where the MFMA pairs it with the fp4 sign taken from bit (j % 32) of the
// canonical word j / 32 (see operand_byte).
constexpr int UP_BLOCK_BYTES = 16 * 128;

// byte offset inside a 128-byte operand column for input column jj (0..127).  The fp4 register s
// of lane group q takes nibble e from native bit 4*e + s, which is column 32*q + 8*s + e, and the
// matrix instruction gives that nibble the contraction index 32*q + 8*s + e: index == column.  Its
// 8-bit operand keeps index k in lane group (k mod 64) / 16, byte (k mod 16) + 16 * (k / 64), so 16
// consecutive columns are 16 consecutive bytes.
__host__ __device__ inline int operand_byte(int jj)
{
    return ((jj & 63) >> 4) * 32 + (jj & 15) + ((jj >> 6) << 4);
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
    int stage_op0;            // first op of the stage this op belongs to
    float sc[2];              // power-of-two input scale per path (max |h| * sc <= 1/2)
    float inv_sc[2];
};

// what a compute wavefront needs to know about an op (copied to LDS)
struct OpInfo {
    uint64_t bits;            // address of the sign tiles
    uint64_t up;              // address of the expanded input
    uint32_t CT;
    uint32_t pad_[3];
};
static_assert(sizeof(OpInfo) == 32, "LDS_INFO_BYTES");

// tiles of one op that one compute wavefront of one workgroup streams (copied to LDS)
struct WaveRec {
    uint32_t tile0;           // first tile, counted from the start of the op's sign array
    uint32_t packed;          // n (tiles, bits 0..15) | ct0 (column tile of the first, 16..23) | slot0 (24..31)
};

struct Stage {
    int op0, nops;            // ops [op0, op0 + nops) are independent of each other
    int wait_before;          // 1: an op of this stage reads what an earlier stage wrote
    int signal_after;         // 1: a later stage reads what this stage writes
};

struct Header {
    int n_ops, n_stages, T, n_groups;
};

// workspace: [Header][Op x n_ops][Stage x n_stages][flags: n_groups x u32][error u32][zero page 128 B]
//            [indices of the ops whose input is expanded by a kernel of its own]
//            [indices of the ops whose input is written by another op of the launch]
//            [OpInfo x n_ops][WaveRec x n_groups x CWAVES x n_ops][up arrays]
struct Layout {
    size_t ops, stages, flags, error, zero, which, poison, info, rec, up, total;
};

__host__ __device__ inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

__host__ __device__ inline size_t up_bytes(int in, int T)
{
    const int CB = (in + 255) / 256 * 2;
    return (size_t)((T + 1) / 2) * CB * UP_BLOCK_BYTES;
}

}  // namespace mx
}  // namespace rb
