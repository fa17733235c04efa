// Matrix-core path: set-up kernels, the persistent stack kernel, and its host
// planner.  See rb_mx.h for the arithmetic and the operand layout.
//
// Work split of the persistent kernel (one workgroup per compute unit):
//   * every op's row tiles are cut into contiguous shares, one per workgroup;
//     a share is a contiguous run of 1 KB sign tiles in the native layout and
//     is cut again into one run per compute wavefront;
//   * what each compute wavefront does is written out once per plan as a list
//     of steps (tile address, operand address, what to do afterwards), so the
//     kernel's loop has no op tables to search;
//   * a compute wavefront keeps RING_D sign tiles in flight from HBM into its
//     LDS ring (the weights of later ops do not depend on activations, so the
//     stream never stops at a stage boundary), reads the expanded input of the
//     current stage NB tiles ahead, and issues four MFMAs per tile;
//   * partial sums of the wavefronts that share a row tile meet in LDS;
//   * four more wavefronts finish rows: y = sum_k g_k * acc_k, fp16 rounding,
//     the store, and the four-term expansion of h (.) y for the ops that read y
//     next, written with device-scope 16-byte stores.  Keeping this traffic on
//     wavefronts of their own means no wait on it ever drains a weight prefetch;
//   * hand-over between compute units: before a launch every 16-byte group of an expanded input
//     that a producer of the launch will write is filled with 0xff bytes, which no bf8 term of a
//     finite value has.  Producers just store.  One finishing wavefront per workgroup announces the
//     next stage to its compute wavefronts a fixed pause after its own stores; a compute wavefront
//     requests operand tiles with plain loads (shared by the 32 compute units of an XCD in its L2)
//     and, when it consumes a tile, checks every 32-bit word of every group; only a tile with a
//     word that still reads 0xffffffff is waited for and read again past the L2.  The pause is a
//     matter of speed, not of correctness.  Device-coherent reads of every operand would put twice
//     the weight traffic on the fabric that also carries the HBM stream.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include <atomic>
#include <cmath>
#include <cstring>
#include <map>
#include <memory>
#include <mutex>
#include <vector>

#include "rabit.h"
#include "rb_internal.h"
#include "rb_layout.h"
#include "rb_mx.h"
#include "rb_mx_device.h"

namespace rb {
namespace mx {


#define RB_LDS(p) ((__attribute__((address_space(3))) void *)(p))
// Pointers read from the op table are generic; dereferencing them as such makes FLAT instructions,
// which also count as LDS traffic: every LDS wait would then wait for global stores to be acknowledged.
#define RB_GLOBAL(T, p) ((__attribute__((address_space(1))) T *)(p))

// Hand-over timing (a matter of speed only: a consuming wavefront checks what it gets).  Pauses are
// in s_sleep units of 64 clocks.
constexpr int GO_PAUSE_1 = 24;      // between a workgroup's own stores and its "go", one token
constexpr int GO_PAUSE_2 = 28;      // ... two tokens
constexpr int TILE_PAUSE_1 = 32;    // per 16 sign tiles that a workgroup is ahead of the busiest one, one token
constexpr int TILE_PAUSE_2 = 44;    // ... two tokens
// between two looks at a tile that was not yet written: the first 64 come quickly, the rest far
// apart (wavefronts that look too often keep the stores they wait for from landing); %[left] counts
// down from 0x40000
#define RB_REPOLL_PAUSE                       \
    "s_sleep 8\n\t"                           \
    "s_cmp_gt_u32 %[left], 0x3ffc0\n\t"       \
    "s_cbranch_scc1 3f\n\t"                   \
    "s_sleep 56\n"                            \
    "3:\n\t"

// ---------------------------------------------------------------- helpers ---
__device__ __forceinline__ uint32_t lds_addr(const void *p)
{
    return (uint32_t)(size_t)RB_LDS(p);
}

// weight of the normalisation in front of the op at input column j (1 where there is none): it is
// folded into the op's input scales
__device__ __forceinline__ float norm_weight(const Op &op, int j)
{
    return op.norm_w ? __half2float(reinterpret_cast<const __half *>(op.norm_w)[j]) : 1.f;
}

// ------------------------------------------------------------ prep kernel ---
// One workgroup per op: power-of-two scale of each path's input scales and the zero fill of the
// expanded-input array (padding columns and unused operand columns must read as zero).
__global__ __launch_bounds__(256) void prep_kernel(Header *hdr, Op *ops, uint32_t *error, uint32_t *zero_page)
{
    const int o = blockIdx.x;
    Op &op = ops[o];
    __shared__ float red[256];
    for (int p = 0; p < op.K; ++p) {
        float m = 0.f;
        for (int j = threadIdx.x; j < op.in; j += 256)
            m = fmaxf(m, fabsf(__half2float(reinterpret_cast<const __half *>(op.h)[(size_t)p * op.in + j]) * norm_weight(op, j)));
        red[threadIdx.x] = m;
        __syncthreads();
        for (int s = 128; s > 0; s >>= 1) {
            if ((int)threadIdx.x < s) red[threadIdx.x] = fmaxf(red[threadIdx.x], red[threadIdx.x + s]);
            __syncthreads();
        }
        if (threadIdx.x == 0) {
            const float sc = input_scale(red[0]);
            op.sc[p] = sc;
            op.inv_sc[p] = 1.f / sc;
        }
        __syncthreads();
    }
    const size_t n16 = up_bytes(op.in, hdr->T) / 16;
    uint4 *up = reinterpret_cast<uint4 *>(op.up);
    for (size_t i = threadIdx.x; i < n16; i += 256) up[i] = make_uint4(0, 0, 0, 0);
    if (o == 0) {
        zero_page[threadIdx.x] = 0;                       // 2 KB: what a padding step of the sign stream reads (up to 1.5 KB)
        zero_page[256 + threadIdx.x] = 0;
        if (threadIdx.x < 2) error[threadIdx.x] = 0;      // the give-up mark and the count of tiles waited for
    }
}

// The step lists of the compute wavefronts; one thread per (workgroup, wavefront).  Row tiles of an
// op are dealt to the workgroups in contiguous, nearly equal shares, and a share (row tiles x column
// tiles, contiguous in the native layout) is cut into one contiguous run per compute wavefront.
// (T is a template argument so that the divisions by the number of compute wavefronts are by a
// constant; the walk over the ops is integer arithmetic from end to end, and runs once per plan)
template <int T>
__global__ __launch_bounds__(64) void desc_kernel(const Header *hdr, const Op *ops, const uint32_t *zero_page,
                                                  uint32_t *sdesc, uint32_t *odesc, uint32_t sblocks, uint32_t oblocks)
{
    // one wavefront per list; its lanes write the entries of an op's run side by side
    const uint32_t G = (uint32_t)hdr->n_groups, id = blockIdx.x, lane = threadIdx.x;
    constexpr uint32_t CW = (uint32_t)cwaves_of(T);
    if (id >= G * CW) return;
    const uint32_t grp = id / CW, wave = id % CW;
    uint32_t *sd = sdesc + (size_t)id * sblocks * (SIGN_FIELDS * DESC_BLOCK);
    uint32_t *od = odesc + (size_t)id * oblocks * (OPND_FIELDS * DESC_BLOCK);
    const uint32_t s_cap = sblocks * DESC_BLOCK, o_cap = oblocks * DESC_BLOCK;
    auto put_sign = [&](uint32_t e, uint64_t addr) {
        if (e >= s_cap) return;
        uint32_t *b = sd + (size_t)(e / DESC_BLOCK) * (SIGN_FIELDS * DESC_BLOCK) + e % DESC_BLOCK;
        b[0] = (uint32_t)addr;
        b[DESC_BLOCK] = (uint32_t)(addr >> 32);
    };
    auto put_opnd = [&](uint32_t e, uint64_t addr, uint32_t meta) {
        if (e >= o_cap) return;
        uint32_t *b = od + (size_t)(e / DESC_BLOCK) * (OPND_FIELDS * DESC_BLOCK) + e % DESC_BLOCK;
        b[0] = (uint32_t)addr;
        b[DESC_BLOCK] = (uint32_t)(addr >> 32);
        b[2 * DESC_BLOCK] = meta;
    };
    uint32_t gs = 0, go = 0;                  // entries written so far (the same in every lane)
    // 64 ops at a time, one op per lane: a lane works out its op's run for this wavefront, a scan
    // over the lanes places the runs one after the other (a stage is a run of consecutive ops and
    // ends with nb_of(T) empty operand entries), and every lane writes the entries of its own op.
    // (A walk op by op costs a few hundred instructions per op and wavefront whether the run has
    // an entry or not: a quarter of a millisecond for a 7B-shaped plan.)
    const int n_ops = hdr->n_ops, K = hdr->K;
    auto share = [&](uint32_t RT, int pos, uint32_t &rt0, uint32_t &nrt) { group_rows(RT, grp, G, pos, rt0, nrt); };
    for (int chunk = 0; chunk < n_ops; chunk += 64) {
        const int o = chunk + (int)lane;
        const bool live = o < n_ops;
        const Op &mo = ops[live ? o : n_ops - 1];
        const uint64_t bits = (uint64_t)mo.bits, up = (uint64_t)mo.up;
        const uint32_t RT = (uint32_t)mo.RT, CT = (uint32_t)mo.CT;
        const int first = mo.stage_op0, dep = mo.dep;
        const bool ends_stage = live && (o == n_ops - 1 || ops[o + 1].stage_op0 != first);
        uint32_t rt0, nrt;
        share(RT, mo.pos, rt0, nrt);
        // first finishing slot of the op: behind the ops of its stage that come before it
        uint32_t slot_base = 0;
        for (int m = first; m < o && live; ++m) {
            uint32_t a, n;
            share((uint32_t)ops[m].RT, ops[m].pos, a, n);
            if (ops[m].slot0 >= 0) slot_base = (uint32_t)ops[m].slot0;
            slot_base += n;
        }
        if (mo.slot0 >= 0) slot_base = (uint32_t)mo.slot0;
        // Run `run` of the share goes to this wavefront.  Runs differ by one tile when CW does not
        // divide the share, and the longer ones sit at the same positions for every op of equal
        // shape; dealing op number n of the stage from wavefront n on spreads them.  The partial
        // sums are filed under the run, not the wavefront, so the order of the final sum is the
        // single-op kernel's whichever wavefront worked on a run.
        const uint32_t run = (wave + (uint32_t)(o - first)) % CW;
        const uint32_t U = nrt * CT, u0 = run * U / CW, u1 = (run + 1) * U / CW;
        const uint32_t n_sign = live ? u1 - u0 : 0u;
        const uint32_t n_opnd = n_sign + (ends_stage ? (uint32_t)nb_of(T) : 0u);
        // where this lane's entries start: exclusive sums over the lanes before it
        uint32_t s_at = n_sign, o_at = n_opnd;
        for (int d = 1; d < 64; d <<= 1) {
            const uint32_t a = __shfl_up(s_at, d), b = __shfl_up(o_at, d);
            if ((int)lane >= d) { s_at += a; o_at += b; }
        }
        const uint32_t s_total = __shfl(s_at, 63), o_total = __shfl(o_at, 63);
        s_at = gs + s_at - n_sign;
        o_at = go + o_at - n_opnd;
        for (uint32_t e = 0; e < n_sign; ++e) {
            const uint32_t u = u0 + e, row = u / CT, ct = u - row * CT, rt = rt0 + row, slot = slot_base + row;
            put_sign(s_at + e, bits + ((size_t)rt * CT + ct) * (size_t)(512 * K));
            put_opnd(o_at + e, up + (size_t)ct * 2 * up_block_bytes(T),
                     STEP_VALID | ((ct == CT - 1 || u == u1 - 1) ? STEP_FLUSH : 0u) | ((slot * CW + run) << STEP_PART_SHIFT) |
                         ((dep >= 0 ? 1u : 0u) << STEP_DEP_SHIFT) | (ct << STEP_CT_SHIFT));
        }
        if (ends_stage)
            for (uint32_t e = 0; e < (uint32_t)nb_of(T); ++e) put_opnd(o_at + n_sign + e, 0, 0u);
        gs += s_total;
        go += o_total;
    }
    // past the last tile: a sign request reads a page of zeros, an operand entry is empty
    for (uint32_t e = gs + lane; e < s_cap; e += 64) put_sign(e, (uint64_t)zero_page);
    for (uint32_t e = go + lane; e < o_cap; e += 64) put_opnd(e, 0, 0u);
}

// Second set-up pass (needs the scales of every op): the tables of the finishing wavefronts.
// One workgroup per (stage, LINK_GROUPS workgroups of the stack kernel); a thread per (slot, row).
constexpr int LINK_GROUPS = 8;
__global__ __launch_bounds__(256) void link_kernel(const Header *hdr, const Op *ops, const Stage *stages,
                                                   SlotRec *slots, float *vals, SlotExt *ext)
{
    const int G = hdr->n_groups, T = hdr->T;
    const int st = blockIdx.x;
    const Stage stage = stages[st];
    // sign tiles of workgroup gg in this stage; the most any workgroup has (all threads take part)
    auto stage_tiles = [&](int gg) {
        uint32_t tiles = 0;
        for (int o = stage.op0; o < stage.op0 + stage.nops; ++o) {
            uint32_t rt0, nrt;
            group_rows((uint32_t)ops[o].RT, (uint32_t)gg, (uint32_t)G, ops[o].pos, rt0, nrt);
            tiles += nrt * (uint32_t)ops[o].CT;
        }
        return tiles;
    };
    __shared__ uint32_t most_of[256];
    uint32_t most = 0;
    for (int gg = threadIdx.x; gg < G; gg += 256) most = max(most, stage_tiles(gg));
    most_of[threadIdx.x] = most;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) most_of[threadIdx.x] = max(most_of[threadIdx.x], most_of[threadIdx.x + s]);
        __syncthreads();
    }
    most = most_of[0];
    // LINK_GROUPS workgroups of the stack kernel per workgroup of this one, two at a time (what a
    // thread reads hangs on a chain of dependent loads: fewer, longer workgroups wait for it less often)
    auto one_group = [&](int grp) {
    if (grp >= G) return;
    const uint32_t mine = stage_tiles(grp);
    const int slot = (threadIdx.x >> 4) & 7, row = threadIdx.x & 15;
    int my_op = -1, row0 = 0, slot_base = 0;
    for (int o = stage.op0; o < stage.op0 + stage.nops; ++o) {
        uint32_t rt0, nrt;
        group_rows((uint32_t)ops[o].RT, (uint32_t)grp, (uint32_t)G, ops[o].pos, rt0, nrt);
        if (ops[o].slot0 >= 0) slot_base = ops[o].slot0;
        if (slot >= slot_base && slot < slot_base + (int)nrt) {
            my_op = o;
            row0 = (int)(rt0 + (uint32_t)(slot - slot_base)) * 16;
        }
        slot_base += (int)nrt;
    }
    if (slot >= stage.n_slots) return;
    const size_t idx = (size_t)stage.rec0 + (size_t)grp * stage.n_slots + slot;
    SlotRec sr;
    sr.y = 0; sr.pad64_ = 0; sr.out = 1; sr.n_cons = 0; sr.row0 = 0; sr.op = -1; sr.pad_ = 0;
    sr.behind = most - mine;
    for (int c = 0; c < MAX_CONS; ++c) sr.up[c] = 0;
    float v[12];
    for (int i = 0; i < 12; ++i) v[i] = 0.f;
    SlotExt sx;
    sx.resid = 0; sx.ssq_in = 0; sx.ssq_out = 0; sx.rcopy = 0; sx.n_part = 0; sx.role = ROLE_PLAIN;
    sx.resid_kind = RESID_NONE; sx.inv_n = 0.f; sx.eps = 0.f; sx.ssq_stride = 0; sx.pad_[0] = sx.pad_[1] = 0;
    if (my_op >= 0) {
        const Op &op = ops[my_op];
        const int grow = row0 + row;
        sx.resid = (uint64_t)op.resid; sx.resid_kind = op.resid_kind;
        sx.ssq_in = (uint64_t)op.ssq_in; sx.n_part = op.ssq_in ? op.n_part : 0;
        sx.ssq_out = op.ssq_out ? (uint64_t)(op.ssq_out + row0 / 16) : 0;
        sx.ssq_stride = op.RT;
        sx.rcopy = (uint64_t)op.rcopy;
        sx.role = op.role; sx.inv_n = 1.f / (float)op.in; sx.eps = op.eps;
        sr.y = (uint64_t)op.y;
        sr.out = op.out; sr.n_cons = op.n_cons; sr.row0 = row0; sr.op = my_op;
        const bool valid = grow < op.out;
        const __half *g = reinterpret_cast<const __half *>(op.g);
        if (valid) {
            v[0] = __half2float(g[grow]) * op.inv_sc[0];
            v[1] = __half2float(g[(size_t)op.out + grow]) * op.inv_sc[1];
            if (op.K == 3) v[8] = __half2float(g[2 * (size_t)op.out + grow]) * op.inv_sc[2];
        }
        for (int c = 0; c < op.n_cons; ++c) {
            const Op &m = ops[op.cons[c]];
            sr.up[c] = (uint64_t)(m.up + up_group_offset(T, row0, 0));
            const __half *h = reinterpret_cast<const __half *>(m.h);
            if (valid) {
                const float w = norm_weight(m, grow);
                v[2 + 2 * c] = __half2float(h[grow]) * w * m.sc[0];
                v[3 + 2 * c] = __half2float(h[(size_t)m.in + grow]) * w * m.sc[1];
                if (m.K == 3) v[9 + c] = __half2float(h[2 * (size_t)m.in + grow]) * w * m.sc[2];
            }
        }
    }
    // 32 bytes per row, 48 with three paths: two or three 16-byte stores
    float4 *vrow = reinterpret_cast<float4 *>(vals + (idx * 16 + (size_t)row) * vals_row_floats(hdr->K));
    vrow[0] = make_float4(v[0], v[1], v[2], v[3]);
    vrow[1] = make_float4(v[4], v[5], v[6], v[7]);
    if (hdr->K == 3) vrow[2] = make_float4(v[8], v[9], v[10], v[11]);
    if (row == 0) {
        slots[idx] = sr;
        if (ext) ext[idx] = sx;
    }
    };
    for (int sub = 0; sub < LINK_GROUPS / 2; ++sub) one_group((int)blockIdx.y * LINK_GROUPS + 2 * sub + (int)(threadIdx.x >> 7));
}

// --------------------------------------------------------- expand kernel ---
// Input scaling u_k = h_k (.) x (Section 4.1) for ops whose input comes from
// outside the fused ops, written as four bf8 terms in operand order.  A thread takes 16 consecutive
// columns of one token and path (in % 32 == 0) and stores one 16-byte group per term.
__device__ __forceinline__ void expand_part(const Header *hdr, const Op *ops, const int *which, int bx, int tok, int bz)
{
    const Op &op = ops[which[bz]];
    const int nblk = op.in / 16;
    const int id = bx * 256 + (int)threadIdx.x;
    if (id >= nblk * op.K) return;
    const int p = id / nblk, j0 = (id - p * nblk) * 16;
    const int T = hdr->T;
    const uint4 *xs = reinterpret_cast<const uint4 *>(op.x + (size_t)tok * op.in + j0);     // buffers are 16-byte aligned
    const uint4 xq[2] = {xs[0], xs[1]};
    const uint32_t xw[8] = {xq[0].x, xq[0].y, xq[0].z, xq[0].w, xq[1].x, xq[1].y, xq[1].z, xq[1].w};
    const __half *hp = reinterpret_cast<const __half *>(op.h) + (size_t)p * op.in + j0;     // scales: 2-byte aligned
    uint32_t out[4][4] = {};                                  // [term][word of the group]
    const float sc = op.sc[p];
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        const float x = __half2float(__ushort_as_half((unsigned short)(xw[e >> 1] >> (16 * (e & 1)))));
        const uint32_t terms = expand4(__half2float(hp[e]) * norm_weight(op, j0 + e) * x * sc);
#pragma unroll
        for (int t = 0; t < 4; ++t) out[t][e >> 2] |= ((terms >> (8 * t)) & 0xffu) << (8 * (e & 3));
    }
    // where path p of this token sits in the layout: three paths use token 1's path 0 for path 2
    const int ltok = op.K == 3 ? p >> 1 : tok, lp = op.K == 3 ? p & 1 : p;
#pragma unroll
    for (int t = 0; t < 4; ++t)
        *reinterpret_cast<uint4 *>(op.up + up_group_offset(T, j0, 8 * ltok + 4 * lp + t)) =
            make_uint4(out[t][0], out[t][1], out[t][2], out[t][3]);
}

// Sums of squares of an input from outside that an op normalises: 16 columns per entry, [token][entry], as the
// finishing wavefronts file them for inputs written inside a launch.  One workgroup per (op, token).
__device__ __forceinline__ void ssq_part(const Op *ops, const int *which, int bx, int tok)
{
    const Op &op = ops[which[bx]];
    if (!op.norm_w || op.dep >= 0) return;
    float *out = const_cast<float *>(op.ssq_in);
    for (int e = threadIdx.x; e < op.n_part; e += 256) {
        float sum = 0.f;
        for (int j = 16 * e; j < min(16 * e + 16, op.in); ++j) {
            const float x = __half2float(reinterpret_cast<const __half *>(op.x)[(size_t)tok * op.in + j]);
            sum += x * x;
        }
        out[(size_t)tok * op.n_part + e] = sum;
    }
}

// Before every launch: the expanded input of every op that a producer of this
// launch will write is set to "not written yet" (0xff in every byte of the 16-byte groups of real
// columns: no bf8 term of a finite value is 0xff; padding columns read as zero).  POISON_SPLIT
// workgroups per op.
constexpr int POISON_SPLIT = 4;
__device__ __forceinline__ void poison_part(const Op *ops, int T, int n_ops, uint4 *aux, size_t aux16, int bx, int by)
{
    if (bx == n_ops) {
        // what finishing wavefronts hand to each other in a decoder block: no sum of squares and
        // no fp16 value in a word of its own is all ones
        for (size_t i = by * 256 + threadIdx.x; i < aux16; i += 256 * POISON_SPLIT)
            aux[i] = make_uint4(0xffffffffu, 0xffffffffu, 0xffffffffu, 0xffffffffu);
        return;
    }
    const Op &op = ops[bx];
    if (op.dep < 0) return;
    const int groups = (int)(up_bytes(op.in, T) / 16);
    uint4 *up = reinterpret_cast<uint4 *>(op.up);
    for (int i = by * 256 + (int)threadIdx.x; i < groups; i += 256 * POISON_SPLIT) {
        // which 16 input columns group i holds (see up_group_offset): a block of 128 columns is
        // [q][half j][operand column 0..7] for one token, [half j][q][operand column 0..15] for two
        // and two such images for four
        const int b = T == 1 ? i >> 6 : T == 2 ? i >> 7 : i >> 8;
        const int q = (i >> 4) & 3;
        const int j = T == 1 ? (i >> 3) & 1 : (i >> 6) & 1;
        const uint32_t v = b * 128 + j * 64 + q * 16 < op.in ? 0xffffffffu : 0u;
        up[i] = make_uint4(v, v, v, v);
    }
}

// What goes before the stack kernel in every run, as one launch: the first n_poison workgroups mark
// inputs (they write the expanded inputs of ops fed from inside the launch), the next n_expand
// expand the inputs from outside (ex x ey x ez workgroups; they write those of the other ops), and
// in a decoder block the rest add up the squares of the inputs from outside that an op normalises
// (one workgroup per such input and token).
__global__ __launch_bounds__(256) void before_kernel(const Header *hdr, const Op *ops, const int *which, int n_poison,
                                                     int n_expand, int ex, int ey, uint4 *aux, size_t aux16)
{
    const int b = (int)blockIdx.x;
    if (b < n_poison) {
        poison_part(ops, hdr->T, hdr->n_ops, aux, aux16, b / POISON_SPLIT, b % POISON_SPLIT);
        return;
    }
    const int e = b - n_poison;
    if (e < n_expand) {
        expand_part(hdr, ops, which, e % ex, (e / ex) % ey, e / (ex * ey));
        return;
    }
    const int q = e - n_expand;
    ssq_part(ops, which, q / ey, q % ey);
}

// ---------------------------------------------------------- stack kernel ---
// workgroup barrier that orders LDS only: the weight prefetch of a compute wavefront stays in
// flight across it (a full fence would wait for every outstanding global load)
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// a store that passes the L2 of this XCD (for another XCD's wavefront to read with a device-scope load)
__device__ __forceinline__ void store_sc1_u32(uint64_t addr, uint32_t v)
{
    asm volatile("global_store_dword %0, %1, off sc1" : : "v"(addr), "v"(v) : "memory");
}
// what a wavefront that gave up a bounded wait leaves in the plan's error word (rb_stack_status
// reports any of them as RB_ERR_HANDOVER; rb_stack_gave_up tells which)
constexpr int GAVE_UP_TILE = 1;       // an input tile was never written
constexpr int GAVE_UP_TORN = 2;       // a tile whose first bytes had arrived kept reading as unwritten
constexpr int GAVE_UP_GO = 3;         // a stage was never announced inside the workgroup
constexpr int GAVE_UP_BLOCK = 4;      // a sum of squares or a residual value of a decoder block never arrived
constexpr uint32_t BLOCK_POLLS = 0x40000;     // looks at a value another workgroup has yet to write, before giving up

__device__ __forceinline__ uint64_t uniform64(uint32_t lo, uint32_t hi)
{
    return ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)hi) << 32) |
           (uint32_t)__builtin_amdgcn_readfirstlane((int)lo);
}

template <int TT> struct BTile { v4i r[kop_of(TT)]; };   // operand of one tile: two 128-column blocks

// What a producer stores carries its own validity (a 16-byte group of an expanded input is all 0xff
// until it is written), so a producer neither waits for its stores to be acknowledged nor raises a
// flag, and nobody polls memory for flags.
// KK = 3 (with TT = 2, the layout; one token of activations): see layout_tokens in rb_mx.h.
// BLK: the form that runs decoder blocks (normalised inputs, gate times up, residual additions in
// the finishing wavefronts; the compute wavefronts are the same).
template <int TT, int KK = 2, bool BLK = false>
__global__ __launch_bounds__(threads_of(TT), 1) void stack_kernel(const Header *__restrict__ hdr_p,
                                                           const Op *__restrict__ ops,
                                                           const Stage *__restrict__ stages,
                                                           uint32_t *__restrict__ error,
                                                           const uint32_t *__restrict__ zero_page,
                                                           const uint32_t *__restrict__ sdesc_g,
                                                           const uint32_t *__restrict__ odesc_g,
                                                           uint32_t sblocks, uint32_t oblocks,
                                                           const SlotRec *__restrict__ slots_g,
                                                           const float *__restrict__ vals_g, int go_pause,
                                                           const SlotExt *__restrict__ ext_g)
{
    static_assert(KK == 2 || (KK == 3 && TT == 2), "three paths use the two-token layout");
    constexpr int CW = cwaves_of(TT), THREADS = threads_of(TT);
    constexpr int TILE_BYTES = 512 * KK, SL = sign_loads_of(KK);
    using Lds = LdsMap<CW, KK, pairs_of(TT)>;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    float *part = reinterpret_cast<float *>(lds + Lds::PART_OFF);

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int grp = blockIdx.x;
    const int n_stages = hdr_p->n_stages;
    constexpr int T = TT, NB = nb_of(TT), KOP = kop_of(TT);

    // ---- LDS set-up: clear the partial sums
    for (int i = threadIdx.x; i < Lds::PART_BYTES / 4; i += THREADS) part[i] = 0.f;
    if (threadIdx.x == 0) *reinterpret_cast<uint32_t *>(lds + Lds::MISC_OFF + WAITED_LDS_OFF) = 0u;
    __syncthreads();

    if (wave < CW) {
        // ======================= compute wavefront ==========================
        uint8_t *const ring = lds + Lds::RING_OFF + wave * (RING_D * TILE_BYTES);
        uint8_t *const ring_end = ring + RING_D * TILE_BYTES;
        const int col = lane & 15, qd = lane >> 4;
        const int scale_b = term_scale(col);
        const uint32_t lane_off = (uint32_t)lane * 16u;
        // diagnostic: every lane of a wavefront that had to wait for a tile adds one here (so 64 per
        // tile); the watching wavefront hands the sum to the workspace at the end
        const uint32_t waited_lds = lds_addr(lds + Lds::MISC_OFF + WAITED_LDS_OFF);
        uint32_t c22;
        asm volatile("v_mov_b32 %0, 0x22222222" : "=v"(c22));
        // A load that carries no data but keeps the number of vector-memory operations per
        // step constant (the in-order completion counter is what the ring relies on): four
        // bytes per lane from the zero page into a scratch corner of LDS.
        uint8_t *dummy_dst = lds + Lds::MISC_OFF + 256 + wave * 256;
        const uint32_t *dummy_src = zero_page;
        auto issue_dummies = [&](int n) {
            for (int i = 0; i < n; ++i) __builtin_amdgcn_global_load_lds(dummy_src, RB_LDS(dummy_dst), 4, 0, 0);
        };
        // ---- the step lists of this wavefront.  Each list is read front to back, a block of 64
        // entries (one per lane) at a time: the wavefront holds the block it reads from and the one
        // after it, and replaces the latter, 64 steps before it is needed, each time it moves on.
        // The replacing loads are written as instructions and never waited for by name: loads
        // complete in order and every step waits for all but its youngest few, so a block has
        // arrived a few steps after its request (steps_done tells when that cannot be relied on).
        const size_t my_list = (size_t)grp * CW + wave;
        const uint32_t *sd_next = sdesc_g + my_list * sblocks * (SIGN_FIELDS * DESC_BLOCK) + lane;
        const uint32_t *od_next = odesc_g + my_list * oblocks * (OPND_FIELDS * DESC_BLOCK) + lane;
        int s_lo, s_hi, sn_lo, sn_hi;                 // sign list: current block, next block
        int o_lo, o_hi, o_m, on_lo, on_hi, on_m;      // operand list
        asm volatile("global_load_dword %0, %10, off\n\t"
                     "global_load_dword %1, %10, off offset:256\n\t"
                     "global_load_dword %2, %10, off offset:512\n\t"
                     "global_load_dword %3, %10, off offset:768\n\t"
                     "global_load_dword %4, %11, off\n\t"
                     "global_load_dword %5, %11, off offset:256\n\t"
                     "global_load_dword %6, %11, off offset:512\n\t"
                     "global_load_dword %7, %11, off offset:768\n\t"
                     "global_load_dword %8, %11, off offset:1024\n\t"
                     "global_load_dword %9, %11, off offset:1280\n\t"
                     "s_waitcnt vmcnt(0)"
                     : "=&v"(s_lo), "=&v"(s_hi), "=&v"(sn_lo), "=&v"(sn_hi), "=&v"(o_lo), "=&v"(o_hi), "=&v"(o_m),
                       "=&v"(on_lo), "=&v"(on_hi), "=&v"(on_m)
                     : "v"(sd_next), "v"(od_next)
                     : "memory");
        sd_next += 2 * SIGN_FIELDS * DESC_BLOCK;
        od_next += 2 * OPND_FIELDS * DESC_BLOCK;
        uint32_t p_sign = 0, p_opnd = 0;              // entries read so far
        uint32_t steps_done = 0, s_mark = 0, o_mark = 0;   // steps consumed; the same at the last block requests
        auto next_sign = [&]() -> uint64_t {
            const int l = (int)(p_sign & (DESC_BLOCK - 1));
            const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane(s_lo, l), hi = (uint32_t)__builtin_amdgcn_readlane(s_hi, l);
            ++p_sign;
            if ((p_sign & (DESC_BLOCK - 1)) == 0) {
                if (steps_done - s_mark < (uint32_t)NB + 2) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                asm volatile("v_mov_b32 %0, %2\n\t"
                             "v_mov_b32 %1, %3\n\t"
                             "global_load_dword %2, %4, off\n\t"
                             "global_load_dword %3, %4, off offset:256"
                             : "=&v"(s_lo), "=&v"(s_hi), "+v"(sn_lo), "+v"(sn_hi)
                             : "v"(sd_next)
                             : "memory");
                sd_next += SIGN_FIELDS * DESC_BLOCK;
                s_mark = steps_done;
            }
            return ((uint64_t)hi << 32) | lo;
        };
        struct OpndDesc { uint32_t lo, hi, meta; };
        auto next_opnd = [&]() -> OpndDesc {
            const int l = (int)(p_opnd & (DESC_BLOCK - 1));
            OpndDesc d;
            d.lo = (uint32_t)__builtin_amdgcn_readlane(o_lo, l);
            d.hi = (uint32_t)__builtin_amdgcn_readlane(o_hi, l);
            d.meta = (uint32_t)__builtin_amdgcn_readlane(o_m, l);
            ++p_opnd;
            if ((p_opnd & (DESC_BLOCK - 1)) == 0) {
                if (steps_done - o_mark < (uint32_t)NB + 2) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                asm volatile("v_mov_b32 %0, %3\n\t"
                             "v_mov_b32 %1, %4\n\t"
                             "v_mov_b32 %2, %5\n\t"
                             "global_load_dword %3, %6, off\n\t"
                             "global_load_dword %4, %6, off offset:256\n\t"
                             "global_load_dword %5, %6, off offset:512"
                             : "=&v"(o_lo), "=&v"(o_hi), "=&v"(o_m), "+v"(on_lo), "+v"(on_hi), "+v"(on_m)
                             : "v"(od_next)
                             : "memory");
                od_next += OPND_FIELDS * DESC_BLOCK;
                o_mark = steps_done;
            }
            return d;
        };
        // the registers of the blocks on their way stay allocated (see keep_operands below)
        auto keep_blocks = [&]() {
            asm volatile("" : "+v"(sn_lo), "+v"(sn_hi), "+v"(on_lo), "+v"(on_hi), "+v"(on_m));
        };

        // ---- sign-tile stream (runs RING_D tiles ahead of the MFMAs, across ops and stages)
        uint8_t *a_slot = ring;
        auto issue_a = [&]() {
            // non-temporal: every sign tile is read once (measured: the stream is ~13% faster)
            const uint64_t addr = next_sign();
            __builtin_amdgcn_global_load_lds(reinterpret_cast<const uint8_t *>(addr) + lane * 16, RB_LDS(a_slot), 16, 0, 2);
            if constexpr (KK == 3) {
                // the last 512 bytes of a 1.5 KB tile: the first 32 lanes (an LDS copy lands at
                // base + 16 * lane whichever lanes take part)
                if (lane < 32)
                    __builtin_amdgcn_global_load_lds(reinterpret_cast<const uint8_t *>(addr) + 1024 + lane * 16,
                                                     RB_LDS(a_slot + 1024), 16, 0, 2);
            }
            a_slot += TILE_BYTES;
            if (a_slot == ring_end) a_slot = ring;
        };

#pragma unroll 1
        for (int d = 0; d < RING_D; ++d) {
            issue_a();
            issue_dummies(KOP);
        }
        uint8_t *c_slot_ptr = ring;           // ring slot of the next tile to consume
        bool failed = false;                  // a producer never delivered: stop waiting, report
        BTile<TT> B[NB];
#pragma unroll
        for (int i = 0; i < NB; ++i)
#pragma unroll
            for (int r = 0; r < KOP; ++r) B[i].r[r] = (v4i){0, 0, 0, 0};
        // Operand loads are written as instructions, so the compiler does not know that their
        // target registers stay busy until the data arrives.  Naming the registers here keeps
        // them allocated (never reused as temporaries) across the code between two stages.
        auto keep_operands = [&]() {
#pragma unroll
            for (int i = 0; i < NB; ++i)
#pragma unroll
                for (int r = 0; r < KOP; ++r) asm volatile("" : "+v"(B[i].r[r]));
        };

        for (int st = 0; st < n_stages; ++st) {
            keep_operands();
            keep_blocks();

            // ---- expanded-input stream of this stage (NB tiles ahead of the MFMAs).  What the
            // consuming step needs to know about a tile travels with it in meta[] (STEP_* fields).
            uint32_t meta[NB], opnd_lo[NB], opnd_hi[NB];      // per ring slot: STEP_* fields and where the tile's operand lives
            auto load_operand = [&](BTile<TT> &dst, v4i rsrc) {
                // The target registers are in-out operands on purpose: the compiler cannot see that
                // a load issued here lands later, and the loads of the last steps of a stage are
                // never waited for.  As in-out operands the registers stay allocated to the operand
                // ring for the whole kernel, so no temporary is ever placed where a late load lands.
                // Plain loads: the flags have shown that these bytes are final, and nobody in
                // this XCD has read them before that, so its L2 holds no older copy.  Each load
                // reads 1 KB of consecutive bytes (the layout of the expanded input sees to that).
                // An empty buffer (no tile) returns zeros without touching memory.  The descriptor's
                // words come out of vector registers (v_readlane) just before; the compiler does not
                // look inside this block, so the wait states a vector-memory instruction needs after
                // such a write are spelled out.
                if constexpr (TT == 1)
                    asm volatile("s_nop 4\n\t"
                                 "buffer_load_dwordx4 %0, %2, %3, 0 offen\n\t"
                                 "buffer_load_dwordx4 %1, %2, %3, 0 offen offset:1024"
                                 : "+v"(dst.r[0]), "+v"(dst.r[1])
                                 : "v"(lane_off), "s"(rsrc)
                                 : "memory");
                else if constexpr (TT == 2)
                    asm volatile("s_nop 4\n\t"
                                 "buffer_load_dwordx4 %0, %4, %5, 0 offen\n\t"
                                 "buffer_load_dwordx4 %1, %4, %5, 0 offen offset:1024\n\t"
                                 "buffer_load_dwordx4 %2, %4, %5, 0 offen offset:2048\n\t"
                                 "buffer_load_dwordx4 %3, %4, %5, 0 offen offset:3072"
                                 : "+v"(dst.r[0]), "+v"(dst.r[1]), "+v"(dst.r[2]), "+v"(dst.r[3])
                                 : "v"(lane_off), "s"(rsrc)
                                 : "memory");
                else {
                    // eight KB: the offset field holds 12 bits, the second half goes through a second address
                    asm volatile("s_nop 4\n\t"
                                 "buffer_load_dwordx4 %0, %8, %10, 0 offen\n\t"
                                 "buffer_load_dwordx4 %1, %8, %10, 0 offen offset:1024\n\t"
                                 "buffer_load_dwordx4 %2, %8, %10, 0 offen offset:2048\n\t"
                                 "buffer_load_dwordx4 %3, %8, %10, 0 offen offset:3072\n\t"
                                 "buffer_load_dwordx4 %4, %9, %10, 0 offen\n\t"
                                 "buffer_load_dwordx4 %5, %9, %10, 0 offen offset:1024\n\t"
                                 "buffer_load_dwordx4 %6, %9, %10, 0 offen offset:2048\n\t"
                                 "buffer_load_dwordx4 %7, %9, %10, 0 offen offset:3072"
                                 : "+v"(dst.r[0]), "+v"(dst.r[1]), "+v"(dst.r[2 % KOP]), "+v"(dst.r[3 % KOP]), "+v"(dst.r[4 % KOP]),
                                   "+v"(dst.r[5 % KOP]), "+v"(dst.r[6 % KOP]), "+v"(dst.r[7 % KOP])
                                 : "v"(lane_off), "v"(lane_off + 4096u), "s"(rsrc)
                                 : "memory");
                }
            };
            // Hand-over: a finishing wavefront of this workgroup announces, with one word in LDS per
            // stage parity, that the inputs of this stage have probably been written.
            const uint32_t go_word = lds_addr(lds + Lds::MISC_OFF) + (uint32_t)((st & 1) * 8);
            auto go_given = [&]() -> bool {
                uint32_t v;
                asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(go_word) : "memory");
                return __builtin_amdgcn_readfirstlane((int)v) != 0;
            };
            // requests the operand of the next entry of the operand list (nothing for an empty entry)
            bool go_seen = false;                             // this stage's inputs have been announced
            auto issue_b = [&](BTile<TT> &dst, uint32_t &m, uint32_t &addr_lo, uint32_t &addr_hi) {
                const OpndDesc d = next_opnd();
                m = d.meta;
                addr_lo = d.lo;
                addr_hi = d.hi & 0xffffu;
                const bool valid = (m & STEP_VALID) != 0;
                const uint32_t dep = (m >> STEP_DEP_SHIFT) & 1u;
                // one announcement per stage
                if (dep != 0 && !go_seen && !failed) {
                    int spins = 0;
                    while (!go_given()) {
                        __builtin_amdgcn_s_sleep(2);
                        if (++spins > (1 << 24)) {
                            failed = true;
                            if (lane == 0) __hip_atomic_store(RB_GLOBAL(uint32_t, error), (uint32_t)GAVE_UP_GO, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            break;
                        }
                    }
                    go_seen = true;
                }
                // raw buffer descriptor: base, stride 0, size (nothing without a tile), 32-bit untyped
                v4i rsrc;
                rsrc[0] = (int)d.lo;
                rsrc[1] = (int)(d.hi & 0xffffu);
                rsrc[2] = valid ? 2 * up_block_bytes(TT) : 0;
                rsrc[3] = 0x00020000;
                load_operand(dst, rsrc);
            };

            v4f acc0 = {0, 0, 0, 0}, acc1 = {0, 0, 0, 0}, acc2 = {0, 0, 0, 0};   // acc2: the third path, or path 0 of tokens 2, 3
            [[maybe_unused]] v4f acc3 = {0, 0, 0, 0};                             // path 1 of tokens 2, 3
            const int parity = st & 1;
            // a quad of lanes holds the four terms of (path = quad & 1, token = quad >> 1); its
            // first lane writes rows 4*qd .. 4*qd+3 of that path and token
            const int quad = col >> 2;
            const uint32_t part_lane = lds_addr(part) + (uint32_t)(parity * MAXSLOT) * Lds::PART_SLOT_BYTES +
                                       (uint32_t)(((quad & 1) * 2 + (quad >> 1)) * 16 + 4 * qd) * 4;
            constexpr int PAIRS = pairs_of(TT);
            auto flush = [&](uint32_t part_index) {       // slot * CW + run: 256 bytes per token pair each
                v4f v;
#pragma unroll
                for (int r = 0; r < 4; ++r) {     // the four lanes of a quad hold terms of the same path
                    // two paths: quad = 2 * token + path.  Three paths: quads 0, 1, 2 are paths 0, 1, 2;
                    // quad 3 takes path 1's signs times columns that are zero
                    const float mine = (quad & 1) ? acc1[r] : (KK == 3 && quad == 2) ? acc2[r] : acc0[r];
                    v[r] = quad_sum(mine);
                }
                if ((col & 3) == 0)
                    asm volatile("ds_write_b128 %0, %1\n\ts_waitcnt lgkmcnt(0)"
                                 :
                                 : "v"(part_lane + part_index * (256u * PAIRS)), "v"(v)
                                 : "memory");
                if constexpr (TT == 4) {          // tokens 2, 3
#pragma unroll
                    for (int r = 0; r < 4; ++r) v[r] = quad_sum((quad & 1) ? acc3[r] : acc2[r]);
                    if ((col & 3) == 0)
                        asm volatile("ds_write_b128 %0, %1\n\ts_waitcnt lgkmcnt(0)"
                                     :
                                     : "v"(part_lane + part_index * (256u * PAIRS) + 256u), "v"(v)
                                     : "memory");
                    acc3 = (v4f){0, 0, 0, 0};
                }
                acc0 = (v4f){0, 0, 0, 0};
                acc1 = (v4f){0, 0, 0, 0};
                acc2 = (v4f){0, 0, 0, 0};
            };

#pragma unroll
            for (int i = 0; i < NB; ++i) { issue_b(B[i], meta[i], opnd_lo[i], opnd_hi[i]); issue_dummies(SL); }

            bool more = true;
            while (more) {
#pragma unroll
                for (int s = 0; s < NB; ++s) {
                    const uint32_t m = meta[s];
                    if (!(m & STEP_VALID)) { more = false; break; }
                    // Every step issues exactly KOP + SL vector-memory loads (the operand loads, the
                    // copies of one sign tile or their stand-ins) and loads complete in order.  The operand of this
                    // tile was requested NB steps ago, followed by wait_of(T) younger loads; the
                    // sign tile is older still (RING_D > NB).  So "at most wait_of(T) outstanding"
                    // means both have arrived.
                    v4u w;
                    uint2 w2 = make_uint2(0u, 0u);                // three paths: words 4 and 5 of the lane's six
                    if constexpr (KK == 2) {
                        asm volatile("s_waitcnt vmcnt(%2)\n\tds_read_b128 %0, %1\n\ts_waitcnt lgkmcnt(0)"
                                     : "=v"(w)
                                     : "v"(lds_addr(c_slot_ptr) + lane * 16), "n"(wait_of(TT, KK))
                                     : "memory");
                    } else {
                        // 24 bytes per lane, 8-byte aligned
                        uint2 wa, wb;
                        asm volatile("s_waitcnt vmcnt(%4)\n\t"
                                     "ds_read_b64 %0, %3\n\t"
                                     "ds_read_b64 %1, %3 offset:8\n\t"
                                     "ds_read_b64 %2, %3 offset:16\n\t"
                                     "s_waitcnt lgkmcnt(0)"
                                     : "=&v"(wa), "=&v"(wb), "=&v"(w2)
                                     : "v"(lds_addr(c_slot_ptr) + lane * 24), "n"(wait_of(TT, KK))
                                     : "memory");
                        w = (v4u){wa.x, wa.y, wb.x, wb.y};
                    }
#pragma unroll
                    for (int r = 0; r < KOP; ++r) asm volatile("" : "+v"(B[s].r[r]));
                    // Each lane holds one 16-byte group per load.  No byte of a written group is 0xff,
                    // so a 32-bit word that reads 0xffffffff has not been written: a tile with such a
                    // word (its producer was late, the L2 of this XCD got hold of the line before it
                    // was written, or a 16-byte store has landed in part) is waited for by looking at
                    // the first word of every group past the L2, and then loaded again whole.  The
                    // look is one statement, so that the operand registers keep their place (a loop
                    // the compiler can see around a reload makes it move them while loads are in flight).
                    auto unwritten_word = [&]() -> bool {
                        bool any = false;
#pragma unroll
                        for (int r = 0; r < KOP; ++r) {
                            const v4i g = B[s].r[r];
                            any |= max(max((uint32_t)g[0], (uint32_t)g[1]), max((uint32_t)g[2], (uint32_t)g[3])) == 0xffffffffu;
                        }
                        return __ballot(any) != 0ull;
                    };
                    if (((m >> STEP_DEP_SHIFT) & 1u) != 0 && !failed && unwritten_word()) {
                        v4i rsrc;
                        rsrc[0] = (int)opnd_lo[s];
                        rsrc[1] = (int)opnd_hi[s];
                        rsrc[2] = 2 * up_block_bytes(TT);
                        rsrc[3] = 0x00020000;
                        // polls until the first byte of every group is written, then holds the tile as
                        // read after that; returns the polls it had left (0: gave up)
                        auto look_again = [&]() -> uint32_t {
                            uint32_t left;
                            unsigned long long unwritten;
                            if constexpr (TT == 1) {
                                int c0, c1;
                                asm volatile("s_mov_b32 %[left], 0x40000\n"
                                             "1:\n\t"
                                             "s_nop 4\n\t"
                                             "buffer_load_dword %[c0], %[off], %[rs], 0 offen sc1\n\t"
                                             "buffer_load_dword %[c1], %[off], %[rs], 0 offen offset:1024 sc1\n\t"
                                             "buffer_load_dwordx4 %[b0], %[off], %[rs], 0 offen sc1\n\t"
                                             "buffer_load_dwordx4 %[b1], %[off], %[rs], 0 offen offset:1024 sc1\n\t"
                                             "s_waitcnt vmcnt(0)\n\t"
                                             "v_and_b32 %[c0], 0xff, %[c0]\n\t"
                                             "v_and_b32 %[c1], 0xff, %[c1]\n\t"
                                             "v_cmp_eq_u32 vcc, 0xff, %[c0]\n\t"
                                             "s_mov_b64 %[un], vcc\n\t"
                                             "v_cmp_eq_u32 vcc, 0xff, %[c1]\n\t"
                                             "s_or_b64 %[un], %[un], vcc\n\t"
                                             "s_cmp_eq_u64 %[un], 0\n\t"
                                             "s_cbranch_scc1 2f\n\t"
                                             RB_REPOLL_PAUSE
                                             "s_sub_u32 %[left], %[left], 1\n\t"
                                             "s_cmp_lg_u32 %[left], 0\n\t"
                                             "s_cbranch_scc1 1b\n"
                                             "2:\n\t"
                                             "v_mov_b32 %[c0], 1\n\t"
                                             "ds_add_u32 %[cnt], %[c0]"
                                             : [b0] "+v"(B[s].r[0]), [b1] "+v"(B[s].r[1]), [c0] "=&v"(c0), [c1] "=&v"(c1),
                                               [un] "=&s"(unwritten), [left] "=&s"(left)
                                             : [off] "v"(lane_off), [rs] "s"(rsrc), [cnt] "v"(waited_lds)
                                             : "vcc", "scc", "memory");
                            } else if constexpr (TT == 4) {
                                // Four tokens: the looks read first words only, and further and further
                                // apart; the tile follows once they all show data.  (A look that fetched
                                // the 8 KB tile as well, from every wavefront that waits, kept the
                                // producers' second store of a row tile from landing for as long as the
                                // looks went on.)
                                int c0, c1, c2, c3, c4, c5, c6, c7;
                                asm volatile("s_mov_b32 %[left], 0x40000\n"
                                             "1:\n\t"
                                             "s_nop 4\n\t"
                                             "buffer_load_dword %[c0], %[off], %[rs], 0 offen sc1\n\t"
                                             "buffer_load_dword %[c1], %[off], %[rs], 0 offen offset:1024 sc1\n\t"
                                             "buffer_load_dword %[c2], %[off], %[rs], 0 offen offset:2048 sc1\n\t"
                                             "buffer_load_dword %[c3], %[off], %[rs], 0 offen offset:3072 sc1\n\t"
                                             "buffer_load_dword %[c4], %[off2], %[rs], 0 offen sc1\n\t"
                                             "buffer_load_dword %[c5], %[off2], %[rs], 0 offen offset:1024 sc1\n\t"
                                             "buffer_load_dword %[c6], %[off2], %[rs], 0 offen offset:2048 sc1\n\t"
                                             "buffer_load_dword %[c7], %[off2], %[rs], 0 offen offset:3072 sc1\n\t"
                                             "s_waitcnt vmcnt(0)\n\t"
                                             "v_and_b32 %[c0], 0xff, %[c0]\n\t"
                                             "v_and_b32 %[c1], 0xff, %[c1]\n\t"
                                             "v_and_b32 %[c2], 0xff, %[c2]\n\t"
                                             "v_and_b32 %[c3], 0xff, %[c3]\n\t"
                                             "v_and_b32 %[c4], 0xff, %[c4]\n\t"
                                             "v_and_b32 %[c5], 0xff, %[c5]\n\t"
                                             "v_and_b32 %[c6], 0xff, %[c6]\n\t"
                                             "v_and_b32 %[c7], 0xff, %[c7]\n\t"
                                             "v_max3_u32 %[c0], %[c0], %[c1], %[c2]\n\t"
                                             "v_max3_u32 %[c3], %[c3], %[c4], %[c5]\n\t"
                                             "v_max3_u32 %[c0], %[c0], %[c3], %[c6]\n\t"
                                             "v_max_u32 %[c0], %[c0], %[c7]\n\t"
                                             "v_cmp_eq_u32 vcc, 0xff, %[c0]\n\t"
                                             "s_mov_b64 %[un], vcc\n\t"
                                             "s_cmp_eq_u64 %[un], 0\n\t"
                                             "s_cbranch_scc1 2f\n\t"
                                             RB_REPOLL_PAUSE
                                             "s_sub_u32 %[left], %[left], 1\n\t"
                                             "s_cmp_lg_u32 %[left], 0\n\t"
                                             "s_cbranch_scc1 1b\n"
                                             "2:\n\t"
                                             "buffer_load_dwordx4 %[b0], %[off], %[rs], 0 offen sc1\n\t"
                                             "buffer_load_dwordx4 %[b1], %[off], %[rs], 0 offen offset:1024 sc1\n\t"
                                             "buffer_load_dwordx4 %[b2], %[off], %[rs], 0 offen offset:2048 sc1\n\t"
                                             "buffer_load_dwordx4 %[b3], %[off], %[rs], 0 offen offset:3072 sc1\n\t"
                                             "buffer_load_dwordx4 %[b4], %[off2], %[rs], 0 offen sc1\n\t"
                                             "buffer_load_dwordx4 %[b5], %[off2], %[rs], 0 offen offset:1024 sc1\n\t"
                                             "buffer_load_dwordx4 %[b6], %[off2], %[rs], 0 offen offset:2048 sc1\n\t"
                                             "buffer_load_dwordx4 %[b7], %[off2], %[rs], 0 offen offset:3072 sc1\n\t"
                                             "s_waitcnt vmcnt(0)\n\t"
                                             "v_mov_b32 %[c0], 1\n\t"
                                             "ds_add_u32 %[cnt], %[c0]"
                                             : [b0] "+v"(B[s].r[0]), [b1] "+v"(B[s].r[1]), [b2] "+v"(B[s].r[2 % KOP]),
                                               [b3] "+v"(B[s].r[3 % KOP]), [b4] "+v"(B[s].r[4 % KOP]), [b5] "+v"(B[s].r[5 % KOP]),
                                               [b6] "+v"(B[s].r[6 % KOP]), [b7] "+v"(B[s].r[7 % KOP]), [c0] "=&v"(c0), [c1] "=&v"(c1),
                                               [c2] "=&v"(c2), [c3] "=&v"(c3), [c4] "=&v"(c4), [c5] "=&v"(c5), [c6] "=&v"(c6),
                                               [c7] "=&v"(c7), [un] "=&s"(unwritten), [left] "=&s"(left)
                                             : [off] "v"(lane_off), [off2] "v"(lane_off + 4096u), [rs] "s"(rsrc), [cnt] "v"(waited_lds)
                                             : "vcc", "scc", "memory");
                            } else {
                                int c0, c1, c2, c3;
                                asm volatile("s_mov_b32 %[left], 0x40000\n"
                                             "1:\n\t"
                                             "s_nop 4\n\t"
                                             "buffer_load_dword %[c0], %[off], %[rs], 0 offen sc1\n\t"
                                             "buffer_load_dword %[c1], %[off], %[rs], 0 offen offset:1024 sc1\n\t"
                                             "buffer_load_dword %[c2], %[off], %[rs], 0 offen offset:2048 sc1\n\t"
                                             "buffer_load_dword %[c3], %[off], %[rs], 0 offen offset:3072 sc1\n\t"
                                             "buffer_load_dwordx4 %[b0], %[off], %[rs], 0 offen sc1\n\t"
                                             "buffer_load_dwordx4 %[b1], %[off], %[rs], 0 offen offset:1024 sc1\n\t"
                                             "buffer_load_dwordx4 %[b2], %[off], %[rs], 0 offen offset:2048 sc1\n\t"
                                             "buffer_load_dwordx4 %[b3], %[off], %[rs], 0 offen offset:3072 sc1\n\t"
                                             "s_waitcnt vmcnt(0)\n\t"
                                             "v_and_b32 %[c0], 0xff, %[c0]\n\t"
                                             "v_and_b32 %[c1], 0xff, %[c1]\n\t"
                                             "v_and_b32 %[c2], 0xff, %[c2]\n\t"
                                             "v_and_b32 %[c3], 0xff, %[c3]\n\t"
                                             "v_cmp_eq_u32 vcc, 0xff, %[c0]\n\t"
                                             "s_mov_b64 %[un], vcc\n\t"
                                             "v_cmp_eq_u32 vcc, 0xff, %[c1]\n\t"
                                             "s_or_b64 %[un], %[un], vcc\n\t"
                                             "v_cmp_eq_u32 vcc, 0xff, %[c2]\n\t"
                                             "s_or_b64 %[un], %[un], vcc\n\t"
                                             "v_cmp_eq_u32 vcc, 0xff, %[c3]\n\t"
                                             "s_or_b64 %[un], %[un], vcc\n\t"
                                             "s_cmp_eq_u64 %[un], 0\n\t"
                                             "s_cbranch_scc1 2f\n\t"
                                             RB_REPOLL_PAUSE
                                             "s_sub_u32 %[left], %[left], 1\n\t"
                                             "s_cmp_lg_u32 %[left], 0\n\t"
                                             "s_cbranch_scc1 1b\n"
                                             "2:\n\t"
                                             "v_mov_b32 %[c0], 1\n\t"
                                             "ds_add_u32 %[cnt], %[c0]"
                                             : [b0] "+v"(B[s].r[0]), [b1] "+v"(B[s].r[1]), [b2] "+v"(B[s].r[2 % KOP]),
                                               [b3] "+v"(B[s].r[3 % KOP]), [c0] "=&v"(c0), [c1] "=&v"(c1), [c2] "=&v"(c2),
                                               [c3] "=&v"(c3), [un] "=&s"(unwritten), [left] "=&s"(left)
                                             : [off] "v"(lane_off), [rs] "s"(rsrc), [cnt] "v"(waited_lds)
                                             : "vcc", "scc", "memory");
                            }
                            return left;
                        };
                        // Each look reads the first word of every group and then, with later loads of
                        // the same wavefront from the same addresses, the groups themselves.  A group
                        // whose store had landed in part is complete one look later; should a word
                        // still read as unwritten after a few more, the run is reported, not trusted.
                        uint32_t reason = look_again() == 0 ? (uint32_t)GAVE_UP_TILE : 0u;
                        for (int again = 0; reason == 0 && unwritten_word(); ++again) {
                            if (again == 4) reason = GAVE_UP_TORN;
                            else if (look_again() == 0) reason = GAVE_UP_TILE;
                        }
                        if (reason != 0) {                    // a producer never delivered: report, stop checking
                            failed = true;
                            if (lane == 0) __hip_atomic_store(RB_GLOBAL(uint32_t, error), reason, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        }
                    }
                    c_slot_ptr += TILE_BYTES;
                    if (c_slot_ptr == ring_end) c_slot_ptr = ring;
                    const BTile<TT> bt = B[s];
                    v8i b0, b1;
                    [[maybe_unused]] v8i c0, c1;                  // four tokens: the operands of tokens 2, 3
                    if constexpr (TT == 1) {
                        // lanes 0..7 of a row of 16 hold the first four registers of their column; the
                        // other four sit eight lanes further on (row_shl:8).  Lanes 8..15 end up with
                        // bytes of no meaning: their columns of the product are never read.
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            b0[i] = bt.r[0][i];
                            b0[4 + i] = __builtin_amdgcn_update_dpp(0, bt.r[0][i], 0x108, 0xf, 0xf, true);
                            b1[i] = bt.r[1][i];
                            b1[4 + i] = __builtin_amdgcn_update_dpp(0, bt.r[1][i], 0x108, 0xf, 0xf, true);
                        }
                    } else if constexpr (TT == 4) {
                        // per 128-column block: the image of tokens 0, 1 (two loads), then that of tokens 2, 3
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            b0[i] = bt.r[0][i]; b0[4 + i] = bt.r[1][i];
                            c0[i] = bt.r[2 % KOP][i]; c0[4 + i] = bt.r[3 % KOP][i];
                            b1[i] = bt.r[4 % KOP][i]; b1[4 + i] = bt.r[5 % KOP][i];
                            c1[i] = bt.r[6 % KOP][i]; c1[4 + i] = bt.r[7 % KOP][i];
                        }
                    } else {
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            b0[i] = bt.r[0][i]; b0[4 + i] = bt.r[1][i];
                            b1[i] = bt.r[2 % KOP][i]; b1[4 + i] = bt.r[3 % KOP][i];
                        }
                    }
                    if constexpr (KK == 2) {
                        // lane words: (columns 0..127: path 0, path 1), (columns 128..255: path 0, path 1)
                        acc0 = mfma_signs(w.x, b0, acc0, c22, scale_b);
                        acc1 = mfma_signs(w.y, b0, acc1, c22, scale_b);
                        acc0 = mfma_signs(w.z, b1, acc0, c22, scale_b);
                        acc1 = mfma_signs(w.w, b1, acc1, c22, scale_b);
                        if constexpr (TT == 4) {
                            acc2 = mfma_signs(w.x, c0, acc2, c22, scale_b);
                            acc3 = mfma_signs(w.y, c0, acc3, c22, scale_b);
                            acc2 = mfma_signs(w.z, c1, acc2, c22, scale_b);
                            acc3 = mfma_signs(w.w, c1, acc3, c22, scale_b);
                        }
                    } else {
                        // (columns 0..127: paths 0, 1, 2), (columns 128..255: paths 0, 1, 2)
                        acc0 = mfma_signs(w.x, b0, acc0, c22, scale_b);
                        acc1 = mfma_signs(w.y, b0, acc1, c22, scale_b);
                        acc2 = mfma_signs(w.z, b0, acc2, c22, scale_b);
                        acc0 = mfma_signs(w.w, b1, acc0, c22, scale_b);
                        acc1 = mfma_signs(w2.x, b1, acc1, c22, scale_b);
                        acc2 = mfma_signs(w2.y, b1, acc2, c22, scale_b);
                    }
                    if (m & STEP_FLUSH) flush((m >> STEP_PART_SHIFT) & 0xffu);
                    ++steps_done;
                    issue_b(B[s], meta[s], opnd_lo[s], opnd_hi[s]);
                    issue_a();
                }
            }
            lds_barrier();                                    // partial sums of the stage are in LDS
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // nothing may land in LDS or registers after the end
        keep_operands();
        keep_blocks();
    } else {
        // ========================= finishing wavefront ======================
        // What a finishing wavefront does after the barrier is on the path from one stage to the
        // next; the three compute wavefronts it shares a SIMD with wake up at the same barrier and
        // would take three of four issue slots for work that then waits for this one anyway.
        __builtin_amdgcn_s_setprio(3);
        const int ew = wave - CW;
        // lane -> (slot, row, token): a wavefront finishes two slots per stage, one per half
        const int half = lane >> 5;
        const int my_slot = ew + EWAVES * half;
        const int row = lane & 15, tok = (lane >> 4) & 1;
        const int tokens = hdr_p->tokens;                 // of the activations (three use the layout of four)

        // Everything a stage's epilogue needs from memory sits in two flat tables indexed by
        // (stage, workgroup, slot) and is requested one stage ahead, while the compute wavefronts
        // work: nothing after the barrier waits for memory.  The loads are unconditional, so the
        // compiler can wait for exactly these and not for younger ones.
        struct Fin {
            SlotRec r;
            v4f a, b, c;                    // the row's values (c: the third path's, when there is one)
            SlotExt x;                      // decoder blocks only
        };
        auto fetch = [&](int st) -> Fin {
            // a slot the stage does not have reads the record of one it has, and is marked unused
            const Stage sg = stages[min(st, n_stages - 1)];
            const size_t idx = (size_t)sg.rec0 + (size_t)grp * sg.n_slots + min(my_slot, sg.n_slots - 1);
            Fin f;
            f.r = slots_g[idx];
            const v4f *pv = reinterpret_cast<const v4f *>(vals_g + (idx * 16 + (size_t)row) * vals_row_floats(KK));
            f.a = pv[0];
            f.b = pv[1];
            if constexpr (KK == 3) f.c = pv[2];
            else f.c = (v4f){0.f, 0.f, 0.f, 0.f};
            if constexpr (BLK) f.x = ext_g[idx];
            if (st >= n_stages || my_slot >= sg.n_slots) f.r.op = -1;
            return f;
        };
        Fin cur = fetch(0);

        const uint32_t ready_lds = lds_addr(lds + Lds::MISC_OFF);
        for (int st = 0; st < n_stages; ++st) {
            const Fin nxt = fetch(st + 1);
            // the go word of the next stage: nobody reads it before this stage's barrier
            if (ew == 0 && lane == 0) {
                const uint32_t a = ready_lds + (uint32_t)(((st + 1) & 1) * 8);
                asm volatile("ds_write_b32 %0, %1" : : "v"(a), "v"(0u) : "memory");
            }
            const bool have_slot = cur.r.op >= 0;
            const int grow = cur.r.row0 + row;
            // ---- decoder blocks: what the epilogue takes from other workgroups' finishing
            // wavefronts is fetched while the compute wavefronts work.  Both are marked "not yet
            // written" (all ones) before the launch and looked at until they are not.
            [[maybe_unused]] float rinv[pairs_of(TT)], radd[pairs_of(TT)];
#pragma unroll
            for (int pr = 0; pr < pairs_of(TT); ++pr) { rinv[pr] = 1.f; radd[pr] = 0.f; }
            if constexpr (BLK) {
                const int tok_in_pair = (TT == 1 || KK == 3) ? 0 : tok;       // three paths: both lanes of a row hold token 0
                // 1 / root mean square of the input, per token: the sums of squares of 16 columns
                // each, added up by the 32 lanes of this slot's half in a fixed order
                const int n_part = have_slot ? cur.x.n_part : 0;
                // the residual stream's values at this lane's row
                const int kind = have_slot && grow < cur.r.out ? cur.x.resid_kind : RESID_NONE;
                if (__any(n_part > 0 || kind != RESID_NONE)) {
                    // not before this stage's inputs have been announced: a look that comes too
                    // early costs a trip to memory and back
                    if (st > 0) {
                        const uint32_t go_word = ready_lds + (uint32_t)((st & 1) * 8);
                        for (int spins = 0; spins < (1 << 22); ++spins) {
                            uint32_t v;
                            asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(go_word) : "memory");
                            if (__builtin_amdgcn_readfirstlane((int)v) != 0) break;
                            __builtin_amdgcn_s_sleep(2);
                        }
                    }
                    v4f tot;
                    // sums of squares come two at a time (their number is even: in % 32 == 0), four
                    // loads per lane in flight
                    const int n2 = n_part >> 1;
                    for (uint32_t left = BLOCK_POLLS;;) {
                        tot = (v4f){0.f, 0.f, 0.f, 0.f};
                        bool unwritten = false;
#pragma unroll
                        for (int t = 0; t < 4; ++t) {
                            if (t < tokens) {
                                const auto *row_t = RB_GLOBAL(const uint64_t, cur.x.ssq_in) + (size_t)t * n2;
                                for (int base = 0; base < n2; base += 128) {
                                    uint64_t two[4];
#pragma unroll
                                    for (int u = 0; u < 4; ++u) {
                                        const int i = base + 32 * u + (lane & 31);
                                        two[u] = i < n2 ? __hip_atomic_load(row_t + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0ull;
                                    }
#pragma unroll
                                    for (int u = 0; u < 4; ++u) {
                                        const uint32_t lo = (uint32_t)two[u], hi = (uint32_t)(two[u] >> 32);
                                        unwritten |= lo == 0xffffffffu || hi == 0xffffffffu;
                                        tot[t] += __uint_as_float(lo) + __uint_as_float(hi);
                                    }
                                }
                            }
                        }
#pragma unroll
                        for (int pr = 0; pr < pairs_of(TT); ++pr) {
                            const int tk = 2 * pr + tok_in_pair;
                            const size_t e = (size_t)tk * cur.r.out + grow;
                            if (kind == RESID_CALLER && tk < tokens) radd[pr] = (float)RB_GLOBAL(_Float16, cur.x.resid)[e];
                            if (kind == RESID_COPY && tk < tokens) {
                                const uint32_t word = __hip_atomic_load(RB_GLOBAL(const uint32_t, cur.x.resid) + e, __ATOMIC_RELAXED,
                                                                        __HIP_MEMORY_SCOPE_AGENT);
                                unwritten |= word == 0xffffffffu;
                                radd[pr] = (float)__builtin_bit_cast(_Float16, (uint16_t)word);
                            }
                        }
                        if (!__any(unwritten)) break;
                        if (--left == 0) {
                            if (lane == 0) __hip_atomic_store(RB_GLOBAL(uint32_t, error), (uint32_t)GAVE_UP_BLOCK, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            break;
                        }
                        // like the looks at a late tile: the first 64 come quickly, the rest far apart
                        __builtin_amdgcn_s_sleep(8);
                        if (left < BLOCK_POLLS - 64) __builtin_amdgcn_s_sleep(56);
                    }
                    // 1 / root mean square of the input, per token: the 32 lanes of this slot's half
                    // add up their shares in a fixed order
                    if (__any(n_part > 0)) {
#pragma unroll
                        for (int m = 1; m < 32; m <<= 1)
#pragma unroll
                            for (int t = 0; t < 4; ++t) tot[t] += __shfl_xor(tot[t], m);
#pragma unroll
                        for (int pr = 0; pr < pairs_of(TT); ++pr) {
                            const int tk = 2 * pr + tok_in_pair;
                            const float sum = tk == 0 ? tot[0] : tk == 1 ? tot[1] : tk == 2 ? tot[2] : tot[3];
                            if (n_part > 0 && tk < tokens) rinv[pr] = rsqrtf(sum * cur.x.inv_n + cur.x.eps);
                        }
                    }
                }
            }
            const int n_cons = have_slot ? cur.r.n_cons : 0;
            // where this lane's partial sums are, worked out before the barrier (what follows it is
            // on the path from the last matrix instruction of the stage to the stores)
            uint32_t p_off = (uint32_t)(((st & 1) * MAXSLOT + my_slot) * CW * (64 * pairs_of(TT)) + (TT == 1 ? 0 : tok * 16) + row);
            asm volatile("" : "+v"(p_off));
            lds_barrier();                                    // partial sums complete
            // One token: the lanes of a row's second-token position are free, so the two lanes of a
            // row split the paths between them (sub = which path) for the sums and the expansion.
            constexpr bool SPLIT = TT == 1;
            const int sub = tok;
            // Three paths: the lane at a row's second-token position stands for path 2 (as that
            // token's path 0, see layout_tokens): its output scale and its readers' input scales
            // are the third path's, and its "path 1" is nothing.
            const bool third = KK == 3 && tok == 1;
            const float g_a = third ? cur.c[0] : cur.a[0], g_b = third ? 0.f : cur.a[1];
            const float hs[MAX_CONS][2] = {{third ? cur.c[1] : cur.a[2], third ? 0.f : cur.a[3]},
                                           {third ? cur.c[2] : cur.b[0], third ? 0.f : cur.b[1]},
                                           {third ? cur.c[3] : cur.b[2], third ? 0.f : cur.b[3]}};
            // this lane's path of each reader's scales (selected value by value: an indexed array
            // would live in scratch memory)
            const float hsub[MAX_CONS] = {sub ? cur.a[3] : cur.a[2], sub ? cur.b[1] : cur.b[0], sub ? cur.b[3] : cur.b[2]};
            // four tokens: the pair of tokens 0, 1, then the pair 2, 3 (this lane's token is 2 * pair + tok)
            constexpr int PAIRS = pairs_of(TT);
#pragma unroll
            for (int pair = 0; pair < PAIRS; ++pair) {
            const bool active = have_slot && (SPLIT || KK == 3 || 2 * pair + tok < tokens) && grow < cur.r.out;
            float yf = 0.f, ysum = 0.f;
            // partial sums of this lane's row: [run][token pair][path][token][row]
            float *P = part + p_off + pair * 64;
            if (active) {
                // sum the partial sums of the runs in run order
                float s0 = 0.f, s1 = 0.f;
                if constexpr (SPLIT) {
                    float mine = 0.f;
#pragma unroll
                    for (int w = 0; w < CW; ++w) mine += P[w * (64 * PAIRS) + sub * 32];
                    const float other = xor16(mine);                // the lane with the same row and the other path
                    s0 = sub ? other : mine;
                    s1 = sub ? mine : other;
                } else {
#pragma unroll
                    for (int w = 0; w < CW; ++w) {
                        s0 += P[w * (64 * PAIRS)];
                        s1 += P[w * (64 * PAIRS) + 32];
                    }
                }
                ysum = path_sum(g_a, s0, g_b, s1);
                if constexpr (KK == 3) ysum += xor16(ysum);                // paths 0 and 1 in one lane of the row, path 2 in the other
            }
            if constexpr (BLK) {
                ysum *= rinv[pair];                                          // the input was x / rms(x) (.) w
                const int role = have_slot ? cur.x.role : ROLE_PLAIN;
                if (__any(role != ROLE_PLAIN)) {
                    // the same rows of the up projection sit in the other half of the wavefront
                    const float other = xor32(ysum);
                    if (role == ROLE_GATE) ysum = ysum / (1.f + __expf(-ysum)) * other;
                }
                ysum += radd[pair];
            }
            _Float16 y16 = (_Float16)0.f;
            const bool writes = active && (KK == 3 ? tok == 0 : (!SPLIT || sub == 0)) && (!BLK || cur.x.role != ROLE_UP);
            const size_t y_at = (size_t)((SPLIT || KK == 3) ? 0 : 2 * pair + tok) * cur.r.out + grow;
            if (active) {
                y16 = (_Float16)ysum;                                        // round to nearest even
                yf = (float)y16;
                // (y itself is stored after what the next stage waits for)
                if constexpr (BLK)
                    if (writes && cur.x.rcopy != 0) store_sc1_u32(cur.x.rcopy + y_at * 4u, (uint32_t)__builtin_bit_cast(uint16_t, y16));
            }
            if constexpr (BLK) {
                // this row tile's sum of squares, for the ops that normalise what they read
                const bool files = have_slot && cur.x.ssq_out != 0;
                if (__any(files)) {
                    const float sq = row_sum(yf * yf);
                    const int tk = (SPLIT || KK == 3) ? 0 : 2 * pair + tok;
                    if (files && row == 0 && ((SPLIT || KK == 3) ? tok == 0 : true) && tk < tokens)
                        store_sc1_u32(cur.x.ssq_out + (uint64_t)tk * (uint32_t)cur.x.ssq_stride * 4u, __float_as_uint(sq));
                }
            }
            // ---- expanded input of the ops that read y next: the term bytes of the 16 rows of a
            // (token, path), one word per lane of a 16-lane row, are transposed in registers into one
            // 16-byte group per term, which lanes 0..3 of the row store.  Rows beyond the end of the
            // matrix give zero bytes (the padding columns of the reader).
            if (have_slot) {
#pragma unroll
                for (int c = 0; c < MAX_CONS; ++c) {
                    if (c < n_cons) {                               // the same in all lanes of the half (two whole rows)
                        uint8_t *const base = reinterpret_cast<uint8_t *>(cur.r.up[c]) + pair * 2048;
                        if constexpr (SPLIT) {
                            const v4i bytes = transpose_16x4_bytes(active ? expand4(hsub[c] * yf) : 0u);
                            uint8_t *dst = base + (4 * sub + row) * 16;
                            if (row < 4) asm volatile("global_store_dwordx4 %0, %1, off sc1" : : "v"(dst), "v"(bytes) : "memory");
                        } else {
#pragma unroll
                            for (int p = 0; p < 2; ++p) {
                                const v4i bytes = transpose_16x4_bytes(active ? expand4(hs[c][p] * yf) : 0u);
                                uint8_t *dst = base + (8 * tok + 4 * p + row) * 16;
                                if (row < 4) asm volatile("global_store_dwordx4 %0, %1, off sc1" : : "v"(dst), "v"(bytes) : "memory");
                            }
                        }
                    }
                }
            }
            if (writes) RB_GLOBAL(_Float16, cur.r.y)[y_at] = y16;
            // clear the partial sums for the stage after next (a run without tiles writes nothing);
            // off the path from the barrier to the stores
            if (active) {
                if constexpr (SPLIT) {
#pragma unroll
                    for (int w = 0; w < CW; ++w) P[w * (64 * PAIRS) + sub * 32] = 0.f;
                } else {
#pragma unroll
                    for (int w = 0; w < CW; ++w) {
                        P[w * (64 * PAIRS)] = 0.f;
                        P[w * (64 * PAIRS) + 32] = 0.f;
                    }
                }
            }
            }   // token pairs
            // ---- tell the compute wavefronts, which may already be in the next stage, when that
            // stage's inputs have probably been written (one wavefront per workgroup)
            if (ew == 0 && st + 1 < n_stages) {
                const uint32_t go_lds = ready_lds + (uint32_t)(((st + 1) & 1) * 8);
                if (stages[st + 1].n_deps != 0) {
                    if (go_pause >= 0) {
                        // a pause given by the caller (tests: none at all, so that nearly every tile is
                        // requested before it is written)
                        for (int i = 0; i < go_pause; ++i) __builtin_amdgcn_s_sleep(1);
                    } else {
                        // the time the slowest producer's stores need to land
                        __builtin_amdgcn_s_sleep(TT == 1 ? GO_PAUSE_1 : GO_PAUSE_2);
                        // a workgroup with a smaller share got here that much before the busiest one,
                        // whose outputs its compute wavefronts would then request too early
                        const uint32_t ahead = (uint32_t)__builtin_amdgcn_readfirstlane((int)cur.r.behind) *
                                               (TT == 1 ? TILE_PAUSE_1 : TILE_PAUSE_2) / 16u;
                        for (uint32_t i = 0; i < ahead; ++i) __builtin_amdgcn_s_sleep(1);
                    }
                }
                if (lane == 0) asm volatile("ds_write_b32 %0, %1" : : "v"(go_lds), "v"(1u) : "memory");
            }
            cur = nxt;
        }
        // after the last barrier no compute wavefront waits for a tile any more
        if (ew == 0 && lane == 0) {
            const uint32_t lanes_waited = *reinterpret_cast<const uint32_t *>(lds + Lds::MISC_OFF + WAITED_LDS_OFF);
            if (lanes_waited != 0)
                __hip_atomic_fetch_add(RB_GLOBAL(uint32_t, error) + 1, lanes_waited / 64u, __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// ------------------------------------------------------------------ host ---
static Layout make_layout(int n_ops, int n_stages, size_t n_records, int n_groups, int cwaves, int K, size_t up_total,
                          size_t sblocks, size_t oblocks, bool block = false, size_t aux_poison = 0, size_t aux_rest = 0)
{
    Layout L;
    size_t o = sizeof(Header);
    o = align_up(o, 128); L.ops = o; o += sizeof(Op) * (size_t)n_ops;
    o = align_up(o, 128); L.stages = o; o += sizeof(Stage) * (size_t)n_stages;
    o = align_up(o, 128); L.error = o; o += 128;
    L.zero = o; o += 2048;
    L.which = o; o += align_up(sizeof(int) * MAX_EXPAND, 128);
    o = align_up(o, 256); L.sdesc = o; o += 4 * SIGN_FIELDS * DESC_BLOCK * sblocks * (size_t)n_groups * (size_t)cwaves;
    o = align_up(o, 256); L.odesc = o; o += 4 * OPND_FIELDS * DESC_BLOCK * oblocks * (size_t)n_groups * (size_t)cwaves;
    o = align_up(o, 128); L.slots = o; o += sizeof(SlotRec) * n_records;
    o = align_up(o, 128); L.vals = o; o += vals_record_bytes(K) * n_records;
    o = align_up(o, 256); L.up = o; o += up_total;
    L.ext = L.aux = o; L.aux_poison = 0;
    if (block) {
        o = align_up(o, 128); L.ext = o; o += sizeof(SlotExt) * n_records;
        o = align_up(o, 256); L.aux = o; o += align_up(aux_poison, 256) + align_up(aux_rest, 256);
        L.aux_poison = align_up(aux_poison, 256);
    }
    L.total = align_up(o, 256);
    return L;
}

int device_groups()
{
    static int cus = 0;
    if (cus == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return 0;
        cus = prop.multiProcessorCount;
    }
    return cus;
}

bool layer_supported(const rb_layer *L, int T)
{
    // three paths: one token (its three paths take the place of two tokens' two paths in the operand)
    return ((L->K == 2 && T >= 1 && T <= MAX_T) || (L->K == 3 && T == 1)) && L->in % 32 == 0 && L->in <= 65536;
}

// per op of a decoder block, at most: sums of squares of its output and of an input from outside,
// and the copy of its output that a later op adds
static size_t block_aux_bound(const rb_layer *layers, int n_layers, int tokens)
{
    size_t most = 0;
    for (int l = 0; l < n_layers; ++l)
        most = std::max(most, align_up((size_t)row_tiles(layers[l].out) * 16, 256) + align_up((size_t)tokens * layers[l].out * 4, 256) +
                                  align_up((size_t)((layers[l].in + 15) / 16) * 16, 256));
    return most;
}

size_t plan_workspace_bytes(const rb_layer *layers, int n_layers, int n_ops, int T_in, bool block)
{
    int T = T_in;
    for (int l = 0; l < n_layers; ++l) T = std::max(T, layout_tokens(T_in, layers[l].K));
    // upper bound: every op could use the widest layer
    size_t up_max = 0;
    for (int l = 0; l < n_layers; ++l) {
        up_max = std::max(up_max, up_bytes(layers[l].in, T));
    }
    int G = device_groups();
    if (G <= 0) G = 1024;  // no device to ask: a bound on compute units
    // steps of one compute wavefront: at most this many per op for the layer with the largest share
    const size_t CW = (size_t)cwaves_of(T);
    size_t per_op = 0;
    for (int l = 0; l < n_layers; ++l) {
        const size_t share = (size_t)((row_tiles(layers[l].out) + G - 1) / G) * col_tiles(layers[l].in);
        per_op = std::max(per_op, (share + CW - 1) / CW + 1);
    }
    const size_t steps = per_op * (size_t)n_ops;
    // slots: a stage holds what its ops need (the two ops of a gate-times-up stage sit at slots s
    // and s + MAXSLOT / 2, which may leave a gap)
    int slots_per_op = 1;
    for (int l = 0; l < n_layers; ++l) slots_per_op = std::max(slots_per_op, (row_tiles(layers[l].out) + G - 1) / G);
    if (block) slots_per_op = std::max(slots_per_op, MAXSLOT / 2);
    slots_per_op = std::min(slots_per_op, MAXSLOT);
    int K = 2;
    for (int l = 0; l < n_layers; ++l) K = std::max(K, layers[l].K);
    return make_layout(n_ops, n_ops, (size_t)n_ops * (size_t)G * (size_t)slots_per_op, G, (int)CW, K, align_up(up_max, 256) * (size_t)n_ops,
                       desc_blocks((uint32_t)(steps + RING_D)), desc_blocks((uint32_t)(steps + (size_t)nb_of(T) * n_ops)),
                       block, block ? block_aux_bound(layers, n_layers, T_in) * (size_t)n_ops : 0, 0)
        .total;
}
size_t plan_workspace_bytes(const rb_layer *layers, int n_layers, int n_ops, int T)
{
    return plan_workspace_bytes(layers, n_layers, n_ops, T, false);
}
// a gate-times-up op of the caller is two ops of the plan
size_t block_workspace_bytes(const rb_layer *layers, int n_layers, int n_ops, int T)
{
    return plan_workspace_bytes(layers, n_layers, 2 * n_ops, T, true);
}

// Host record of a prepared plan, keyed by the workspace that holds its device part.
struct Prepared {
    Layout lay;
    int n_ops = 0, n_stages = 0, G = 0, T = 0, K = 2, tokens = 0, max_expand_in = 0, n_expand = 0;   // T: of the operand layout
    uint32_t sblocks = 0, oblocks = 0;      // blocks per step list of a compute wavefront
    bool chained = false;                   // some op reads what another op of the launch writes
    bool block = false;                     // a decoder block: the kernel form with the epilogues
    bool ext_norm = false;                  // some op normalises an input from outside
    // host memory the plan's tables are copied from: pageable, so it must outlive the queued copies
    std::shared_ptr<std::vector<uint8_t>> blob;
    std::shared_ptr<std::vector<int>> which;
};
// pause between a workgroup's stores and its announcement of the next stage, in clocks (< 0: the
// built-in timing); see rb_stack_set_option
static std::atomic<int> g_pause_clks{-1};
void set_pause(int clks) { g_pause_clks.store(clks < 0 ? -1 : std::min(clks, 1 << 18)); }
static std::mutex g_mutex;
static std::map<const void *, Prepared> g_prepared;

// one op of a plan: a layer between two buffers and, in a decoder block, what surrounds it
struct PlanOp {
    int layer, src, dst;      // dst < 0: the result leaves through another op (ROLE_UP)
    int norm;                 // >= 0: which weight vector normalises the input
    int add;                  // >= 0: the buffer added to the result
    int role;
};

static int prepare_any(const rb_layer *layers, const PlanOp *sops, int n_ops, uint16_t *const *bufs,
                       const uint16_t *const *norm_w, float eps, bool block, int tokens, void *workspace,
                       size_t workspace_bytes_, hipStream_t stream)
{
    const int G = device_groups();
    if (G <= 0) return RB_ERR_HIP;
    if (block && tokens > MAX_T) return RB_ERR_UNSUPPORTED;
    // one kernel form per plan: every op has the same number of paths
    const int K = layers[sops[0].layer].K;
    for (int n = 0; n < n_ops; ++n)
        if (layers[sops[n].layer].K != K || !layer_supported(&layers[sops[n].layer], tokens)) return RB_ERR_UNSUPPORTED;
    if (block && K == 3 && tokens != 1) return RB_ERR_UNSUPPORTED;
    const int T = layout_tokens(tokens, K);            // tokens of the operand layout

    // ---- ops, consumers, stages
    std::vector<Op> ops((size_t)n_ops);
    std::vector<int> expand_list;
    size_t up_total = 0;
    std::vector<size_t> up_off((size_t)n_ops);
    std::vector<bool> need_ssq((size_t)n_ops, false), need_rcopy((size_t)n_ops, false);
    std::vector<int> resid_from((size_t)n_ops, -1);
    for (int n = 0; n < n_ops; ++n) {
        const rb_layer &L = layers[sops[n].layer];
        Op &o = ops[(size_t)n];
        std::memset(&o, 0, sizeof(Op));
        o.bits = static_cast<const uint32_t *>(L.bits);
        o.g = L.g; o.h = L.h;
        o.x = bufs[sops[n].src];
        o.y = sops[n].dst >= 0 ? bufs[sops[n].dst] : nullptr;
        o.slot0 = -1;
        o.role = sops[n].role;
        o.norm_w = sops[n].norm >= 0 ? norm_w[sops[n].norm] : nullptr;
        o.eps = eps;
        o.out = L.out; o.in = L.in; o.K = L.K;
        o.RT = row_tiles(L.out); o.CT = col_tiles(L.in);
        up_off[(size_t)n] = up_total;
        up_total += align_up(up_bytes(L.in, T), 256);
        // producer of this op's input: the last earlier op that writes the same buffer
        int producer = -1;
        for (int m = n - 1; m >= 0; --m)
            if (sops[m].dst == sops[n].src) { producer = m; break; }
        o.dep = producer;
        if (o.norm_w) {
            o.n_part = (L.in + 15) / 16;
            if (producer >= 0) need_ssq[(size_t)producer] = true;
        }
        // what is added: the caller's buffer as it was before the launch, or what an earlier op wrote there
        if (sops[n].add >= 0) {
            int writer = -1;
            for (int m = n - 1; m >= 0; --m)
                if (sops[m].dst == sops[n].add) { writer = m; break; }
            if (writer >= 0) {
                if (ops[(size_t)writer].out != L.out) return RB_ERR_SHAPE;
                need_rcopy[(size_t)writer] = true;
                resid_from[(size_t)n] = writer;
                o.resid_kind = RESID_COPY;
            } else {
                o.resid = bufs[sops[n].add];
                o.resid_kind = RESID_CALLER;
            }
        }
        if (producer < 0) {
            o.expand_x = 1;
            expand_list.push_back(n);
        } else {
            Op &pr = ops[(size_t)producer];
            if (pr.n_cons >= MAX_CONS) return RB_ERR_UNSUPPORTED;
            if (pr.out != o.in) return RB_ERR_SHAPE;
            pr.cons[pr.n_cons++] = n;
        }
    }
    if (expand_list.size() > MAX_EXPAND || n_ops > MAX_OPS) return RB_ERR_UNSUPPORTED;
    std::vector<Stage> stages;
    size_t n_records = 0;
    {
        int op0 = 0;
        while (op0 < n_ops) {
            Stage s{};
            s.op0 = op0;
            int slots = 0;
            for (int n = op0; n < n_ops; ++n) {
                bool conflict = false;
                for (int m = op0; m < n; ++m) {
                    if (sops[m].dst < 0 || sops[n].dst < 0) continue;
                    if (sops[m].dst == sops[n].src || sops[m].dst == sops[n].dst || sops[m].src == sops[n].dst ||
                        sops[m].dst == sops[n].add || sops[m].add == sops[n].dst)
                        conflict = true;
                }
                const int per_group = (ops[(size_t)n].RT + G - 1) / G;
                if (per_group > MAXSLOT) return RB_ERR_UNSUPPORTED;
                if (sops[n].role == ROLE_GATE) {
                    // gate and up: a stage of their own; the row tiles of the two are dealt alike and
                    // finish in the two halves of the same wavefronts (slots s and s + 4)
                    if (n > op0) break;
                    if (per_group > MAXSLOT / 2) return RB_ERR_UNSUPPORTED;
                    ops[(size_t)n].slot0 = 0;
                    ops[(size_t)n + 1].slot0 = MAXSLOT / 2;
                    if (ops[(size_t)n].dep >= 0) s.n_deps += 2;
                    s.nops = 2;
                    slots = MAXSLOT / 2 + per_group;
                    break;
                }
                if (conflict || slots + per_group > MAXSLOT) break;
                ops[(size_t)n].pos = n - op0;
                if (ops[(size_t)n].dep >= 0) ++s.n_deps;
                slots += per_group;
                ++s.nops;
            }
            s.n_slots = slots;
            s.rec0 = (uint32_t)n_records;
            n_records += (size_t)G * (size_t)slots;
            stages.push_back(s);
            op0 += s.nops;
        }
    }
    for (const Stage &st : stages)
        for (int n = st.op0; n < st.op0 + st.nops; ++n) ops[(size_t)n].stage_op0 = st.op0;
    Prepared pr;
    pr.n_ops = n_ops; pr.n_stages = (int)stages.size(); pr.G = G; pr.T = T; pr.K = K; pr.tokens = tokens;
    pr.n_expand = (int)expand_list.size();
    for (int n : expand_list) pr.max_expand_in = std::max(pr.max_expand_in, ops[(size_t)n].in);
    for (int n = 0; n < n_ops; ++n) pr.chained = pr.chained || ops[(size_t)n].dep >= 0 || resid_from[(size_t)n] >= 0;
    // an upper bound on the step list of a compute wavefront: the largest share of every op, cut in
    // CW runs, rounded up (the exact maximum over workgroups and wavefronts costs more host time than
    // the few blocks it saves)
    {
        const size_t CW = (size_t)cwaves_of(T);
        size_t longest = 0;
        for (int n = 0; n < n_ops; ++n) {
            const size_t share = (size_t)((ops[(size_t)n].RT + G - 1) / G) * (size_t)ops[(size_t)n].CT;
            longest += (share + CW - 1) / CW;
        }
        // entries a wavefront reads: every tile's, plus the look-ahead past the end
        pr.sblocks = desc_blocks((uint32_t)(longest + RING_D));
        pr.oblocks = desc_blocks((uint32_t)(longest + (size_t)nb_of(T) * (size_t)pr.n_stages));
    }
    // decoder blocks: what finishing wavefronts hand to each other (marked unwritten before every
    // launch), then the sums of squares of inputs from outside
    std::vector<size_t> ssq_off((size_t)n_ops, 0), rcopy_off((size_t)n_ops, 0), ext_off((size_t)n_ops, 0);
    size_t aux_poison = 0, aux_rest = 0;
    for (int n = 0; n < n_ops && block; ++n) {
        if (need_ssq[(size_t)n]) { ssq_off[(size_t)n] = aux_poison; aux_poison += align_up((size_t)ops[(size_t)n].RT * 16, 256); }
        if (need_rcopy[(size_t)n]) { rcopy_off[(size_t)n] = aux_poison; aux_poison += align_up((size_t)tokens * ops[(size_t)n].out * 4, 256); }
        if (ops[(size_t)n].norm_w && ops[(size_t)n].dep < 0) {
            ext_off[(size_t)n] = aux_rest;
            aux_rest += align_up((size_t)ops[(size_t)n].n_part * 16, 256);
            pr.ext_norm = true;
        }
    }
    pr.block = block;
    if (n_records > 0xffffffffull) return RB_ERR_UNSUPPORTED;
    pr.lay = make_layout(n_ops, pr.n_stages, n_records, G, cwaves_of(T), K, up_total, pr.sblocks, pr.oblocks, block, aux_poison,
                         aux_rest);
    const Layout &lay = pr.lay;
    if (workspace_bytes_ < lay.total) return RB_ERR_WORKSPACE;
    uint8_t *ws = static_cast<uint8_t *>(workspace);
    for (int n = 0; n < n_ops; ++n) ops[(size_t)n].up = ws + lay.up + up_off[(size_t)n];
    for (int n = 0; n < n_ops && block; ++n) {
        Op &o = ops[(size_t)n];
        if (need_ssq[(size_t)n]) o.ssq_out = reinterpret_cast<float *>(ws + lay.aux + ssq_off[(size_t)n]);
        if (need_rcopy[(size_t)n]) o.rcopy = reinterpret_cast<uint32_t *>(ws + lay.aux + rcopy_off[(size_t)n]);
    }
    for (int n = 0; n < n_ops && block; ++n) {
        Op &o = ops[(size_t)n];
        if (o.norm_w)
            o.ssq_in = o.dep >= 0 ? ops[(size_t)o.dep].ssq_out
                                  : reinterpret_cast<const float *>(ws + lay.aux + lay.aux_poison + ext_off[(size_t)n]);
        if (resid_from[(size_t)n] >= 0) o.resid = ops[(size_t)resid_from[(size_t)n]].rcopy;
    }

    Header hdr{};
    hdr.n_ops = n_ops; hdr.n_stages = pr.n_stages; hdr.T = T; hdr.n_groups = G; hdr.K = K; hdr.tokens = tokens;

    // ---- upload: stream-ordered copies out of host memory that the plan's record keeps alive
    pr.blob = std::make_shared<std::vector<uint8_t>>(lay.error, (uint8_t)0);
    std::vector<uint8_t> &blob = *pr.blob;
    std::memcpy(blob.data(), &hdr, sizeof(hdr));
    std::memcpy(blob.data() + lay.ops, ops.data(), sizeof(Op) * (size_t)n_ops);
    std::memcpy(blob.data() + lay.stages, stages.data(), sizeof(Stage) * (size_t)pr.n_stages);
    pr.which = std::make_shared<std::vector<int>>(expand_list);
    const int *which = pr.which->data();
    if (hipMemcpyAsync(ws, blob.data(), lay.error, hipMemcpyHostToDevice, stream) != hipSuccess) return RB_ERR_HIP;
    if (!expand_list.empty() &&
        hipMemcpyAsync(ws + lay.which, which, sizeof(int) * expand_list.size(), hipMemcpyHostToDevice, stream) !=
            hipSuccess)
        return RB_ERR_HIP;
    {
        std::lock_guard<std::mutex> lock(g_mutex);
        g_prepared[workspace] = pr;
    }
    hipLaunchKernelGGL(prep_kernel, dim3(n_ops), dim3(256), 0, stream, reinterpret_cast<Header *>(ws),
                       reinterpret_cast<Op *>(ws + lay.ops),
                       reinterpret_cast<uint32_t *>(ws + lay.error), reinterpret_cast<uint32_t *>(ws + lay.zero));
    auto lists = [&](auto kernel) {
        hipLaunchKernelGGL(kernel, dim3(G * cwaves_of(T)), dim3(64), 0, stream, reinterpret_cast<const Header *>(ws),
                           reinterpret_cast<const Op *>(ws + lay.ops), reinterpret_cast<const uint32_t *>(ws + lay.zero),
                           reinterpret_cast<uint32_t *>(ws + lay.sdesc), reinterpret_cast<uint32_t *>(ws + lay.odesc), pr.sblocks,
                           pr.oblocks);
    };
    if (T == 1) lists(desc_kernel<1>);
    else if (T == 2) lists(desc_kernel<2>);
    else lists(desc_kernel<4>);
    hipLaunchKernelGGL(link_kernel, dim3(pr.n_stages, (G + LINK_GROUPS - 1) / LINK_GROUPS), dim3(256), 0, stream,
                       reinterpret_cast<const Header *>(ws), reinterpret_cast<const Op *>(ws + lay.ops),
                       reinterpret_cast<const Stage *>(ws + lay.stages), reinterpret_cast<SlotRec *>(ws + lay.slots),
                       reinterpret_cast<float *>(ws + lay.vals), block ? reinterpret_cast<SlotExt *>(ws + lay.ext) : nullptr);
    return hipGetLastError() == hipSuccess ? RB_OK : RB_ERR_HIP;
}

int prepare_plan(const rb_layer *layers, const rb_stack_op *sops, int n_ops, uint16_t *const *bufs, int tokens,
                 void *workspace, size_t workspace_bytes_, hipStream_t stream)
{
    std::vector<PlanOp> pops((size_t)n_ops);
    for (int n = 0; n < n_ops; ++n) pops[(size_t)n] = PlanOp{sops[n].layer, sops[n].src, sops[n].dst, -1, -1, ROLE_PLAIN};
    return prepare_any(layers, pops.data(), n_ops, bufs, nullptr, 0.f, false, tokens, workspace, workspace_bytes_, stream);
}

int prepare_block(const rb_layer *layers, const uint16_t *const *norm_w, float eps, const rb_block_op *bops, int n_bops,
                  uint16_t *const *bufs, int tokens, void *workspace, size_t workspace_bytes_, hipStream_t stream)
{
    std::vector<PlanOp> pops;
    for (int n = 0; n < n_bops; ++n) {
        const rb_block_op &b = bops[n];
        if (b.epilogue == RB_EPI_SILU_MUL) {
            pops.push_back(PlanOp{b.layer, b.src, b.dst, b.norm, -1, ROLE_GATE});
            pops.push_back(PlanOp{b.aux, b.src, -1, b.norm, -1, ROLE_UP});
        } else {
            pops.push_back(PlanOp{b.layer, b.src, b.dst, b.norm, b.epilogue == RB_EPI_ADD ? b.aux : -1, ROLE_PLAIN});
        }
    }
    return prepare_any(layers, pops.data(), (int)pops.size(), bufs, norm_w, eps, true, tokens, workspace, workspace_bytes_,
                       stream);
}

int launch_plan(void *workspace, size_t workspace_bytes_, hipStream_t stream)
{
    Prepared pr;
    {
        std::lock_guard<std::mutex> lock(g_mutex);
        const auto it = g_prepared.find(workspace);
        if (it == g_prepared.end()) return RB_ERR_WORKSPACE;
        pr = it->second;
    }
    if (workspace_bytes_ < pr.lay.total) return RB_ERR_WORKSPACE;
    uint8_t *ws = static_cast<uint8_t *>(workspace);
    const Layout &lay = pr.lay;
    Header *d_hdr = reinterpret_cast<Header *>(ws);
    Op *d_ops = reinterpret_cast<Op *>(ws + lay.ops);
    const int n_poison = pr.chained ? (pr.n_ops + (lay.aux_poison ? 1 : 0)) * POISON_SPLIT : 0;
    const int ex = (pr.max_expand_in / 16 * RB_MAX_K + 255) / 256, ey = pr.tokens;
    const int n_expand_groups = pr.n_expand > 0 ? ex * ey * pr.n_expand : 0;
    const int n_ssq_groups = pr.ext_norm ? pr.n_expand * ey : 0;
    if (n_poison + n_expand_groups + n_ssq_groups > 0)
        hipLaunchKernelGGL(before_kernel, dim3((unsigned)(n_poison + n_expand_groups + n_ssq_groups)), dim3(256), 0, stream, d_hdr,
                           d_ops, reinterpret_cast<const int *>(ws + lay.which), n_poison, n_expand_groups, ex, ey,
                           reinterpret_cast<uint4 *>(ws + lay.aux), lay.aux_poison / 16);
    const int pause_clks = g_pause_clks.load();
    const int go_pause = pause_clks < 0 ? -1 : pause_clks / 64;      // s_sleep units
    auto launch = [&](auto kernel, int threads, int lds_bytes) -> int {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                lds_bytes) != hipSuccess)
            return RB_ERR_HIP;
        hipLaunchKernelGGL(kernel, dim3(pr.G), dim3(threads), lds_bytes, stream, d_hdr, d_ops,
                           reinterpret_cast<const Stage *>(ws + lay.stages),
                           reinterpret_cast<uint32_t *>(ws + lay.error), reinterpret_cast<const uint32_t *>(ws + lay.zero),
                           reinterpret_cast<const uint32_t *>(ws + lay.sdesc), reinterpret_cast<const uint32_t *>(ws + lay.odesc),
                           pr.sblocks, pr.oblocks,
                           reinterpret_cast<const SlotRec *>(ws + lay.slots), reinterpret_cast<const float *>(ws + lay.vals),
                           go_pause, pr.block ? reinterpret_cast<const SlotExt *>(ws + lay.ext) : nullptr);
        return RB_OK;
    };
    const int rc = pr.block    ? (pr.K == 3   ? launch(stack_kernel<2, 3, true>, threads_of(2), LdsMap<cwaves_of(2), 3>::BYTES)
                                  : pr.T == 1 ? launch(stack_kernel<1, 2, true>, threads_of(1), LdsMap<cwaves_of(1)>::BYTES)
                                  : pr.T == 2 ? launch(stack_kernel<2, 2, true>, threads_of(2), LdsMap<cwaves_of(2)>::BYTES)
                                              : launch(stack_kernel<4, 2, true>, threads_of(4), LdsMap<cwaves_of(4), 2, 2>::BYTES))
                   : pr.K == 3 ? launch(stack_kernel<2, 3>, threads_of(2), LdsMap<cwaves_of(2), 3>::BYTES)
                   : pr.T == 1 ? launch(stack_kernel<1>, threads_of(1), LdsMap<cwaves_of(1)>::BYTES)
                   : pr.T == 2 ? launch(stack_kernel<2>, threads_of(2), LdsMap<cwaves_of(2)>::BYTES)
                               : launch(stack_kernel<4>, threads_of(4), LdsMap<cwaves_of(4), 2, 2>::BYTES);
    if (rc != RB_OK) return rc;
    return hipGetLastError() == hipSuccess ? RB_OK : RB_ERR_HIP;
}

int plan_status(const void *workspace, hipStream_t stream, unsigned long long *waited, int *reason)
{
    Prepared pr;
    {
        std::lock_guard<std::mutex> lock(g_mutex);
        const auto it = g_prepared.find(workspace);
        if (it == g_prepared.end()) return RB_ERR_WORKSPACE;
        pr = it->second;
    }
    uint32_t mark[2] = {0, 0};               // gave up a wait; tiles waited for
    if (hipMemcpyAsync(mark, static_cast<const uint8_t *>(workspace) + pr.lay.error, sizeof(mark), hipMemcpyDeviceToHost,
                       stream) != hipSuccess ||
        hipStreamSynchronize(stream) != hipSuccess)
        return RB_ERR_HIP;
    if (waited) *waited += mark[1];
    if (reason && mark[0]) *reason = (int)mark[0];
    return mark[0] ? RB_ERR_HANDOVER : RB_OK;
}

void forget_plan(const void *workspace)
{
    std::lock_guard<std::mutex> lock(g_mutex);
    g_prepared.erase(workspace);
}

int run_plan(const rb_layer *layers, const rb_stack_op *sops, int n_ops, uint16_t *const *bufs, int T,
             void *workspace, size_t workspace_bytes_, hipStream_t stream)
{
    const int rc = prepare_plan(layers, sops, n_ops, bufs, T, workspace, workspace_bytes_, stream);
    if (rc != RB_OK) return rc;
    return launch_plan(workspace, workspace_bytes_, stream);
}

}  // namespace mx
}  // namespace rb
