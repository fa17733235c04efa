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

// ---- roles of the sixteen wavefronts of a workgroup of the persistent kernel (one per compute unit)
constexpr int NL = 2;              // stream sign tiles from HBM into the LDS ring
constexpr int NC = 12;             // consume tiles: sign expansion and matrix instructions
constexpr int NF = 2;              // finish rows: sums, scales, rounding, stores, expansion for the readers
constexpr int WAVES = NL + NC + NF;
constexpr int THREADS = WAVES * 64;
static_assert(WAVES == 16, "one workgroup of 1024 threads per compute unit");

constexpr int RING_TILES = 128;    // sign tiles (1 KB each) the LDS ring of a compute unit holds
constexpr int MAX_SLOTS = 2 * NF;  // row tiles one compute unit finishes per phase (a finishing wavefront takes two)
constexpr int NPAR = 2;            // phases whose partial sums LDS holds at once
constexpr int MAX_CONS = 3;        // ops that read one op's output inside a fused stack
constexpr int MAX_T = 2;           // tokens per launch on this path
constexpr int MAX_OPS = 4096;      // ops per launch
constexpr size_t MAX_EXPAND = 1024;
constexpr int LOADER_WINDOW = 12;  // sign tiles a loading wavefront keeps in flight (at most 48: see its wait for a free slot)

// ---- how a row tile's contraction is cut into partial sums.  The cut depends on the width of the
// matrix only - not on the number of compute units, of wavefronts, or on how a plan splits an op
// into phases - so that a layer gives the same bits wherever and however it is scheduled: a chunk
// is chunk_tiles(CT) consecutive column tiles accumulated in order from zero, and the chunks of a
// row are added in order.
constexpr int MAX_CHUNKS = 12;
__host__ __device__ constexpr int chunk_tiles(int CT) { return (CT + MAX_CHUNKS - 1) / MAX_CHUNKS; }
__host__ __device__ constexpr int chunks_of(int CT) { return (CT + chunk_tiles(CT) - 1) / chunk_tiles(CT); }

// operand tiles (expanded input of one sign tile) a consuming wavefront requests ahead
constexpr int nb_of(int T) { return T == 1 ? 3 : 2; }
// 16-byte loads per lane that bring in the operand of one tile
constexpr int kop_of(int T) { return T == 1 ? 2 : 4; }

// LDS map of the persistent kernel for T tokens
template <int T> struct LdsMap {
    static constexpr int RING_BYTES = RING_TILES * 1024;
    static constexpr int PART_ENTRY = T * 2 * 16 * 4;                     // [path][token][row] fp32
    static constexpr int PART_BYTES = NPAR * MAX_SLOTS * MAX_CHUNKS * PART_ENTRY;
    static constexpr int STAGE_WAVE = 2 * MAX_CONS * T * 2 * 4 * 16;      // [half][reader][token][path][term][row] bytes
    static constexpr int STAGE_BYTES = NF * STAGE_WAVE;
    static constexpr int CTRL_BYTES = 256;
    static constexpr int RING_OFF = 0;
    static constexpr int PART_OFF = RING_OFF + RING_BYTES;
    static constexpr int STAGE_OFF = PART_OFF + PART_BYTES;
    static constexpr int CTRL_OFF = STAGE_OFF + STAGE_BYTES;
    static constexpr int BYTES = CTRL_OFF + CTRL_BYTES;
    static_assert(BYTES <= 160 * 1024, "LDS of one compute unit");
};
// control words (uint32) at CTRL_OFF
constexpr int CTRL_LANDED = 0;       // [NL] sign tiles each loading wavefront has brought in (8-byte aligned pair)
constexpr int CTRL_CONSUMED = 2;     // sign tiles of completed phases (ring space that may be reused)
constexpr int CTRL_FAILED = 3;       // a bounded wait ran out somewhere in this workgroup
constexpr int CTRL_WAITED = 4;       // operand tiles found unwritten and read again
constexpr int CTRL_FIN = 6;          // [NF] phases each finishing wavefront has completed (8-byte aligned pair)
constexpr int CTRL_DONE = 8;         // [NPAR] consuming wavefronts that are through with a phase of this parity (running total)
constexpr int CTRL_FIN_TIME = 16;    // [8] clock at which the outputs of phase (index mod 8) were stored
static_assert(NL == 2 && NF == 2, "the pairs above are read with one 8-byte load");

// Expanded input ("right operand") of one op, stored as the register image the MFMA wants, so
// that one load instruction of a wavefront reads 1 KB of consecutive bytes (16 per lane).
// The 8-bit right operand of v_mfma_scale_f32_16x16x128_f8f6f4 keeps, in lane col + 16 * q
// (col = operand column, q = 0..3), contraction indices 16q..16q+15 in its first four registers and
// 64+16q..64+16q+15 in the next four.  Contraction index == input column inside a 128-column block
// (see rb_layout.h), and the operand column is 8 * token + 4 * path + term.
//   two tokens:  block b is 2 KB: [half j of the contraction][lane col + 16q][16 bytes]
//   one token:   only columns 0..7 exist, so block b is 1 KB: [q][j][col][16 bytes]; lane
//                col + 16q of the load gets (j = col / 8, column col % 8), i.e. lanes 0..7 of each
//                row of 16 hold the first four registers of their column, and the next four
//                registers come from eight lanes further on with one cross-lane move each.
// A 16-byte group is the 16 input columns one row tile of the producing op writes.
__host__ __device__ constexpr int up_block_bytes(int T) { return T == 1 ? 1024 : 2048; }

// byte offset of the 16-byte group of (input column block of 16 starting at j0, operand column c)
__host__ __device__ inline size_t up_group_offset(int T, int j0, int c)
{
    const int b = j0 >> 7, jj = j0 & 127, q = (jj & 63) >> 4, j = jj >> 6;
    return T == 1 ? (size_t)b * 1024 + (size_t)(q * 16 + j * 8 + c) * 16
                  : (size_t)b * 2048 + (size_t)j * 1024 + (size_t)(q * 16 + c) * 16;
}

__host__ __device__ inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

__host__ __device__ inline size_t up_bytes(int in, int T)
{
    const int CB = (in + 255) / 256 * 2;           // whole column tiles: two blocks each
    return (size_t)CB * up_block_bytes(T);
}

struct Op {
    const uint32_t *bits;     // native sign tiles
    const uint16_t *g;        // fp16 [K][out]
    const uint16_t *h;        // fp16 [K][in]
    const uint16_t *x;        // fp16 [T][in]  input buffer (read by the expansion kernel only)
    uint16_t *y;              // fp16 [T][out] output buffer
    uint8_t *up;              // expanded input of this op (see up_group_offset)
    int out, in;
    int RT, CT;               // row tiles (16 rows), column tiles (256 columns)
    int n_cons;               // ops that read y inside this call
    int cons[MAX_CONS];
    int expand_x;             // 1: x comes from outside the fused ops and must be expanded first
    int dep;                  // op of this launch that writes x (-1: none)
    int last_phase;           // the phase that completes this op's output
    float sc[2];              // power-of-two input scale per path (max |h| * sc in [1/4, 1/2))
    float inv_sc[2];
};

// A phase is a range of row tiles of one op, dealt to the workgroups in contiguous shares; the
// phases of a plan run in order on every compute unit, without a barrier between them.  What the
// planner writes (host):
struct PhaseSeed {
    int op, rt_first, n_rt, rot;       // rot: the workgroup that gets the first share
};
// ... and what the kernel reads, complete with everything the finishing wavefronts need about the
// op and the ops that read its output (uniform loads, no table look-ups on the way to the stores):
struct Reader {
    uint64_t up;              // expanded input of the reading op
    uint64_t h;               // its input scales, fp16 [2][in]
    float sc[2];              // its power-of-two input scale per path
    int in, pad_;
};
struct Phase {
    uint64_t bits, up, y, g;
    int out, CT, rt_first, n_rt;
    int dep_phase;            // phase that completes this op's input (-1: complete before the launch)
    int n_cons;
    float inv_sc[2];
    int chunk, n_chunks;      // column tiles per partial sum; partial sums per row tile
    int up_bytes, op;
    Reader cons[MAX_CONS];
    int pad_[8];
};
static_assert(sizeof(Reader) == 32 && sizeof(Phase) == 208, "read with scalar loads");

// the share of phase p that workgroup grp owns: row tiles [rt0, rt0 + nrt)
struct Share {
    int rt0, nrt;
};

// What a consuming wavefront does is written out once per plan as the list of its units, in plan
// order, so that its loop decodes one small record per unit instead of working out shares, chunks
// and sequence numbers per phase, and so that it can request the expanded input of the units to
// come while it still works on the present one.  A unit is a chunk of one row tile: `tiles`
// consecutive sign tiles starting at number `seq0` of the workgroup's tile sequence (the ring slot
// follows from it), against the expanded input that starts `up_off` bytes into the plan's array of
// expanded inputs; its partial sums go to entry `part` of the partial-sum area.
struct Unit {
    uint32_t seq0;
    uint32_t up_off;
    uint32_t w2;              // tiles | part << UNIT_PART_SHIFT | UNIT_LAST: the wavefront's last unit of its phase
    uint32_t w3;              // phase | (1 + phase that completes the input, 0: complete before the launch) << 16
};
constexpr int UNIT_PART_SHIFT = 8;
constexpr uint32_t UNIT_LAST = 1u << 20;
static_assert(NPAR * MAX_SLOTS * MAX_CHUNKS < 4096, "twelve bits for the partial-sum entry");
constexpr int MAX_PHASES = 65535;   // sixteen bits in a unit record

struct Header {
    int n_ops, n_phases, T, n_groups;
    int unit_stride;          // unit records per consuming wavefront (the last one used is an end mark: no tiles)
    int pad_[3];
};

// workspace: [Header][Op x n_ops][PhaseSeed x n_phases][error u32 x 2 ...][indices of the ops
//            whose input a kernel of its own expands][Phase x n_phases][Share x n_phases x n_groups]
//            [Unit x unit_stride x NC x n_groups][expanded inputs]
struct Layout {
    size_t ops, seeds, error, which, phases, shares, units, up, total;
};

}  // namespace mx
}  // namespace rb
