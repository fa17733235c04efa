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

// Wavefronts that stream weights and issue MFMAs.  One compute unit holds one workgroup of at
// most 16 wavefronts; what a step costs is instruction issue, so more wavefronts per SIMD help as
// long as the registers suffice: twelve for one token (128 registers each), eight for two.
constexpr int cwaves_of(int T) { return T == 1 ? 12 : 8; }
constexpr int MAX_CWAVES = 12;
static_assert(cwaves_of(1) <= MAX_CWAVES && cwaves_of(2) <= MAX_CWAVES, "sizes of per-wavefront tables");
constexpr int EWAVES = 4;          // wavefronts that finish rows and talk to other CUs
constexpr int threads_of(int T) { return (cwaves_of(T) + EWAVES) * 64; }
constexpr int RING_D = 6;           // sign tiles requested ahead per compute wavefront (1 KB each)
// expanded-input operands requested ahead per compute wavefront (tiles); each holds 8 registers per
// lane for one token and 16 for two.  Measured on the 7B-shaped stack: depths 2 to 8 stream equally
// fast without dependencies between the ops; with them, a request made later is less often made
// before its producer has written (2 against 4: -1.5 % per token, -2.7 % for two tokens), and one
// tile ahead no longer hides the latency (+9 %).
constexpr int nb_of(int T) { return T == 1 ? 2 : 2; }
// vector-memory loads per step: operand loads (16 bytes per lane each) and one sign tile
constexpr int kop_of(int T) { return T == 1 ? 2 : T == 2 ? 4 : 8; }
// copies that bring in one sign tile (1 KB each; a three-path tile is 1.5 KB)
constexpr int sign_loads_of(int K) { return K == 3 ? 2 : 1; }
// Loads complete in order.  The operand of a tile is requested nb steps before its use, the sign
// tile RING_D > nb steps before; when at most this many loads are outstanding both have arrived.
constexpr int wait_of(int T, int K) { return (nb_of(T) - 1) * (kop_of(T) + sign_loads_of(K)) + sign_loads_of(K); }
constexpr int MAXSLOT = 8;         // (op, row tile) pairs one CU finishes per stage
constexpr int MAX_CONS = 3;        // ops that read one op's output inside a fused stack
constexpr int MAX_T = 4;           // tokens per launch on this path
// Four tokens are two pairs: every 128-column block of the expanded input holds the two-token
// operand of tokens 0, 1 and then that of tokens 2, 3; a sign tile is expanded once and multiplied
// with both.  Three tokens use the same layout with the last token's columns left zero.
constexpr int pairs_of(int T) { return T == 4 ? 2 : 1; }
constexpr int MAX_OPS = 4096;      // ops per launch
constexpr size_t MAX_EXPAND = 1024;
static_assert(RING_D > nb_of(1) && RING_D > nb_of(2) && RING_D > nb_of(4) && wait_of(1, 2) <= 63 && wait_of(2, 2) <= 63 &&
                  wait_of(2, 3) <= 63 && wait_of(4, 2) <= 63,
              "the in-order wait counts on this");
// Three paths, one token, ride on the two-token machinery: the 16 operand columns are 8 * token +
// 4 * path + term for two paths; a three-path op puts its paths 0 and 1 where token 0 has them and
// its path 2 where token 1 has path 0 (columns 8..11); columns 12..15 are zero.  LAYOUT_T is the
// token count of the operand layout, not of the activations.
constexpr int layout_tokens(int T, int K) { return K == 3 ? 2 : T == 3 ? 4 : T; }

// LDS map of the stack kernel with CW compute wavefronts
template <int CW, int K = 2, int PAIRS = 1> struct LdsMap {
    static constexpr int RING_BYTES = CW * RING_D * 512 * K;
    // partial sums: [parity][slot][compute wavefront][token pair][path][token of the pair][row] fp32
    static constexpr int PART_SLOT_BYTES = CW * PAIRS * 2 * 2 * 16 * 4;
    static constexpr int PART_BYTES = 2 * MAXSLOT * PART_SLOT_BYTES;
    // go words and a counter, per-wavefront target of the stand-in loads
    static constexpr int MISC_BYTES = 256 + CW * 256;
    static constexpr int RING_OFF = 0;
    static constexpr int PART_OFF = RING_OFF + RING_BYTES;
    static constexpr int MISC_OFF = PART_OFF + PART_BYTES;
    static constexpr int BYTES = MISC_OFF + MISC_BYTES;
    static_assert(BYTES <= 160 * 1024, "LDS of one compute unit");
};

// Expanded input ("right operand") of one op, stored as the register image the MFMA wants, so
// that one load instruction of a wavefront reads 1 KB of consecutive bytes (16 per lane).
// The 8-bit right operand of v_mfma_scale_f32_16x16x128_f8f6f4 keeps, in lane col + 16 * q
// (col = operand column, q = 0..3), contraction indices 16q..16q+15 in its first four registers and
// 64+16q..64+16q+15 in the next four.  Contraction index == input column inside a 128-column block
// (see rb_layout.h), and the operand column is 8 * token + 4 * path + term.
//   two tokens:  block b is 2 KB: [half j of the contraction][lane col + 16q][16 bytes]
//   four tokens: block b is 4 KB: the two-token image of tokens 0, 1, then that of tokens 2, 3
//                (operand column 8 * token + 4 * path + term runs to 31; its bit 4 picks the image)
//   one token:   only columns 0..7 exist, so block b is 1 KB: [q][j][col][16 bytes]; lane
//                col + 16q of the load gets (j = col / 8, column col % 8), i.e. lanes 0..7 of each
//                row of 16 hold the first four registers of their column, and the next four
//                registers come from eight lanes further on with one cross-lane move each.
// A 16-byte group is the 16 input columns one row tile of the producing op writes.
__host__ __device__ constexpr int up_block_bytes(int T) { return T == 1 ? 1024 : T == 2 ? 2048 : 4096; }

// byte offset of the 16-byte group of (input column block of 16 starting at j0, operand column c)
__host__ __device__ inline size_t up_group_offset(int T, int j0, int c)
{
    const int b = j0 >> 7, jj = j0 & 127, q = (jj & 63) >> 4, j = jj >> 6;
    return T == 1   ? (size_t)b * 1024 + (size_t)(q * 16 + j * 8 + c) * 16
           : T == 2 ? (size_t)b * 2048 + (size_t)j * 1024 + (size_t)(q * 16 + c) * 16
                    : (size_t)b * 4096 + (size_t)(c >> 4) * 2048 + (size_t)j * 1024 + (size_t)(q * 16 + (c & 15)) * 16;
}

struct Op {
    const uint32_t *bits;     // native sign tiles
    const uint16_t *g;        // fp16 [K][out]
    const uint16_t *h;        // fp16 [K][in]
    const uint16_t *x;        // fp16 [T][in]  input buffer (read by the expansion kernel only)
    uint16_t *y;              // fp16 [T][out] output buffer
    uint8_t *up;              // expanded input of this op (see up_group_offset)
    int out, in, K;
    int RT, CT;               // row tiles (16 rows), column tiles (256 columns)
    int n_cons;               // ops that read y inside this call
    int cons[MAX_CONS];
    int expand_x;             // 1: x comes from outside the fused ops and must be expanded first
    int dep;                  // op of this launch that writes x (-1: none)
    int stage_op0;            // first op of the stage this op belongs to
    float sc[RB_MAX_K];       // power-of-two input scale per path (max |h| * sc <= 1/2)
    float inv_sc[RB_MAX_K];
    // ---- the decoder block around the layer (all unused, zero, in a plain stack)
    int pos;                  // which rotation of the workgroups the row tiles are dealt by (position in the stage)
    int slot0;                // first finishing slot of this op in every workgroup (< 0: right after the op before it)
    int role;                 // ROLE_*
    int resid_kind;           // RESID_*
    const uint16_t *norm_w;   // fp16 [in]: the input is normalised (root mean square) and multiplied by this
    const float *ssq_in;      // [4][n_part]: per token, sums of squares of 16 input rows each
    float *ssq_out;           // [4][RT]: the same of this op's output, for readers that normalise it
    uint32_t *rcopy;          // [T][out]: the fp16 output once more, one word each, for an op that adds it later
    const void *resid;        // what is added to the result: fp16 [T][out] of the caller or another op's rcopy
    int n_part;
    float eps;
};
// the gate and the up projection of a feed-forward part run as two ops of one stage whose row tiles
// meet in the two halves of a finishing wavefront: y = silu(gate) * up leaves through the gate op
constexpr int ROLE_PLAIN = 0, ROLE_GATE = 1, ROLE_UP = 2;
constexpr int RESID_NONE = 0, RESID_CALLER = 1, RESID_COPY = 2;

// What a compute wavefront does, step by step (one step = one 1 KB sign tile), written out once per
// plan so that the kernel's loop is a walk over two lists and not a search through op tables:
//   sign list:    the address of each tile, in the order the wavefront meets them (requested
//                 RING_D steps ahead, across stages)
//   operand list: per stage, one entry per tile (the address of the tile's expanded input and what
//                 to do after the MFMAs) followed by nb_of(T) empty entries; the first empty entry
//                 that reaches the front of the operand ring ends the stage
// A list is stored in blocks of 64 entries, field by field (64 low words, 64 high words, ...), so
// that a wavefront loads a block with one dword load per field, an entry per lane, and picks the
// entry of a step out of its registers.
constexpr int DESC_BLOCK = 64;               // entries per block (one per lane)
constexpr int SIGN_FIELDS = 2;               // address low, high
constexpr int OPND_FIELDS = 3;               // address low, high, STEP_* fields
constexpr uint32_t STEP_VALID = 1u;          // a tile (empty entries are all zero)
constexpr uint32_t STEP_FLUSH = 2u;          // last tile of its row tile for this wavefront: write the partial sums
constexpr int STEP_PART_SHIFT = 8;           // 8 bits: where the partial sums go: slot * cwaves_of(T) + run of the share
constexpr int STEP_DEP_SHIFT = 16;           // 1 bit: the input is written by an op of this launch (0: it was complete before)
constexpr int STEP_CT_SHIFT = 20;            // 12 bits: column tile
// blocks a wavefront may load for a list of n entries read front to back: it holds the block it
// reads from and the one after it
__host__ __device__ constexpr uint32_t desc_blocks(uint32_t n) { return n / DESC_BLOCK + 2; }

// What a finishing wavefront needs for finishing slot `slot` of workgroup `grp` in stage `st`
// (one row tile of one op), laid out flat: record stages[st].rec0 + grp * stages[st].n_slots + slot,
// so that its address follows from the stage's entry and (grp, slot) alone and nothing on the path
// from the partial sums to the stores waits for a chain of dependent loads.
struct SlotRec {
    uint64_t y;               // fp16 output: row 0 of token 0
    uint64_t pad64_;
    uint64_t up[MAX_CONS];    // per reading op: the 16-byte group of operand column 0 these rows fill
    int out, n_cons;          // rows of the op; ops that read its output
    int row0, op;             // first row of the row tile; op index (< 0: slot unused)
    uint32_t behind;          // sign tiles the busiest workgroup of this stage has more than this one
    uint32_t pad_;
};
static_assert(sizeof(SlotRec) == 64, "four 16-byte loads");
// per row of the slot: g_1 / sc_1, g_2 / sc_2 of the op (its output scales over the input scaling
// it was fed with), then h_k * sc_k (k = 1, 2) of each reading op (its input scales times its input
// scaling); for three paths g_3 / sc_3 and the readers' h_3 * sc_3 follow
// (eight floats per row for two paths, twelve for three; a record is 16 rows)
__host__ __device__ constexpr int vals_row_floats(int K) { return K == 3 ? 12 : 8; }
__host__ __device__ constexpr size_t vals_record_bytes(int K) { return (size_t)16 * vals_row_floats(K) * sizeof(float); }
static_assert(8 >= 2 + 2 * MAX_CONS && 12 >= 3 + 3 * MAX_CONS, "32 or 48 bytes per row");

// More per slot, read only by the form of the kernel that runs decoder blocks.
struct SlotExt {
    uint64_t resid;           // element (token 0, row 0 of the op) of what is added to the result
    uint64_t ssq_in;          // sums of squares of the input, [4][n_part]
    uint64_t ssq_out;         // this row tile's entry of the op's own sums of squares (0: nobody reads them)
    uint64_t rcopy;           // element (token 0, row 0) of the op's copy of its output (0: none)
    int n_part, role, resid_kind;
    float inv_n, eps;         // 1 / in
    int ssq_stride;           // entries per token of the op's own sums of squares
    int pad_[2];
};
static_assert(sizeof(SlotExt) == 64, "four 16-byte loads");

struct Stage {
    int op0, nops;            // ops [op0, op0 + nops) are independent of each other
    int n_deps;               // ops of this stage whose input an earlier stage of the launch writes
    int n_slots;              // finishing slots a workgroup may use in this stage (the tables hold that many per workgroup)
    uint32_t rec0;            // index of the stage's first record in the slot tables
    int pad_[3];
};
static_assert(sizeof(Stage) == 32, "two 16-byte loads");
// First 256 bytes of the miscellaneous LDS area: one "go" word per stage parity at bytes 0 and 8
// (set = the inputs of that stage have probably been written), and a counter.
constexpr int WAITED_LDS_OFF = 240;   // lanes that waited for a tile not yet written

struct Header {
    int n_ops, n_stages, T, n_groups;     // T: tokens of the operand layout (layout_tokens)
    int K, tokens;                        // paths; tokens of the activations
    int pad_[2];
};

// workspace: [Header][Op x n_ops][Stage x n_stages][error u32][zero page 1 KB]
//            [indices of the ops whose input is expanded by a kernel of its own]
//            [sign lists, operand lists: blocks x n_groups x cwaves_of(T) each]
//            [SlotRec x records][value records x the same][up arrays]   (records: see Stage)
//            decoder blocks: [SlotExt x the same][sums of squares and output copies of ops]
//                            [sums of squares of inputs from outside]
struct Layout {
    size_t ops, stages, error, zero, which, sdesc, odesc, slots, vals, up, ext, aux, total;
    size_t aux_poison;        // bytes at the start of aux that every launch marks as not yet written
};

__host__ __device__ inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

__host__ __device__ inline size_t up_bytes(int in, int T)
{
    const int CB = (in + 255) / 256 * 2;           // whole column tiles: two blocks each
    return (size_t)CB * up_block_bytes(T);
}

}  // namespace mx
}  // namespace rb
