// Small-batch path of the residual-binary layer (3 to 16 tokens, and any batch up to 16 for three
// paths): every op of a stack streams its packed weights ONCE for all tokens.
//
// Section 4.1: Y[t] = sum_k g_k (.) (B_k (h_k (.) X[t])).  The arithmetic is the one of the decode
// kernels (rb_mx.h): signs as fp4 +-1 left operands of v_mfma_scale_f32_16x16x128_f8f6f4, the
// scaled input u_k = h_k (.) x as a sum of four bf8 terms in the right operand.  What differs is
// the shape of the work:
//   * the 16 columns of a right operand are 4 tokens x 4 terms of ONE path, so a sign tile costs
//     K * ceil(T / 4) * 2 matrix instructions and its sign expansion is done once for all tokens;
//   * the right operands of a column tile (4 KB per path and group of four tokens) are staged in
//     LDS and shared by the sixteen wavefronts of a workgroup; the staging of the next column
//     tile overlaps the matrix instructions of the present one;
//   * a workgroup owns R row tiles (16 rows each) and all columns: wavefront (r, s) takes row tile
//     r and every S-th of the 2 K (128-column half, path) pieces of a sign tile, R * S = 16.  The
//     partial sums of the S wavefronts of a row tile meet in LDS, where the workgroup adds them in
//     a fixed order, rounds to fp16, stores Y and writes the expanded input of the ops that read
//     Y.  Nothing is exchanged between workgroups, so a launch needs no counters, no scratch
//     memory and no device-scope traffic; an op of 4096 rows is 64 workgroups, which at these
//     sizes (a few hundred KB per workgroup) is bound by launch and memory latency, not by the
//     number of compute units it covers;
//   * the ops of a stack that do not depend on each other (q/k/v, gate/up of a transformer block)
//     run in one launch; ops that depend on each other are ordered by the stream.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include <algorithm>
#include <atomic>
#include <cstring>
#include <map>
#include <memory>
#include <mutex>
#include <vector>

#include "rabit.h"
#include "rb_internal.h"
#include "rb_layout.h"
#include "rb_mx_device.h"

namespace rb {
namespace batch {

using mx::v4f;
using mx::v4i;
using mx::v8i;
typedef unsigned v2u __attribute__((ext_vector_type(2)));

constexpr int MAX_T = 16;
constexpr int MAX_CONS = 3;            // ops that read one op's output inside a stack
constexpr int WAVES = 16;              // wavefronts of a workgroup
constexpr int THREADS = WAVES * 64;
constexpr int MAX_STAGE_OPS = 8;       // independent ops that share a launch
// S wavefronts share P row tiles, each taking every S-th piece (128-column half x path) of their
// sign tiles; a workgroup owns R = 16 / S * P row tiles.  Few row tiles per workgroup make many
// workgroups out of a small op; many row tiles share the staged right operands among more rows,
// which is what counts when a launch has workgroups enough anyway (at 16 tokens the operands of a
// column tile are 32 KB, a sign tile 1 KB).  With P = 2 a wavefront reads an operand from LDS once
// for two matrix instructions: at 16 tokens the reads of the operands, 2 KB per instruction, are
// what a compute unit spends most of a column tile on.  The form is chosen per launch (see
// prepare_plan): two paths (S, P) = (2, 2), (4, 2) or (4, 1), i.e. 16, 8 or 4 row tiles per
// workgroup; three paths (2, 1) (two row tiles of three paths would need 96 accumulator registers
// at 16 tokens).
struct Form { int S, P; };
__host__ __device__ constexpr int n_forms(int K) { return K == 2 ? 3 : 1; }
__host__ __device__ constexpr Form form_of(int K, int i)     // by falling row tiles per workgroup
{
    return K == 2 ? (i == 0 ? Form{2, 2} : i == 1 ? Form{4, 2} : Form{4, 1}) : Form{2, 1};
}
__host__ __device__ constexpr int block_tiles(int S, int P) { return WAVES / S * P; }      // row tiles of a workgroup
constexpr int WANT_GROUPS = 256;       // workgroups a launch should have before it takes larger row blocks
constexpr size_t MAX_EXPAND = 1024;

#define RB_LDS(p) ((__attribute__((address_space(3))) void *)(p))
// Pointers read from the op table are generic; dereferencing them as such makes FLAT instructions,
// which may touch LDS as far as the hardware and the compiler know: every one of them would wait
// for all copies into LDS that are still in flight.
#define RB_GLOBAL(T, p) ((__attribute__((address_space(1))) T *)(p))

__host__ __device__ constexpr int groups_of(int T) { return (T + 3) / 4; }
// bytes of the right operands of one column tile: [128-column block][path][token group] x 2 KB,
// each the register image the matrix instruction wants: [half j of the contraction][lane col + 16 q][16 bytes]
__host__ __device__ constexpr size_t tile_operand_bytes(int K, int G) { return (size_t)2 * K * G * 2048; }
__host__ __device__ inline size_t operand_bytes(int in, int K, int G) { return (size_t)col_tiles(in) * tile_operand_bytes(K, G); }
// byte offset of the 16-byte group (16 consecutive input columns starting at j0, path k, token
// group g, operand column c = 4 * (token % 4) + term)
__host__ __device__ inline size_t operand_group_offset(int K, int G, int j0, int k, int g, int c)
{
    const int b = j0 >> 7, jj = j0 & 127, q = (jj & 63) >> 4, j = jj >> 6;
    return ((size_t)(b * K + k) * G + g) * 2048 + (size_t)j * 1024 + (size_t)(q * 16 + c) * 16;
}

struct Reader {
    uint8_t *up;              // expanded input of the reading op
    const uint16_t *h;        // its input scales, fp16 [K][in]
    float sc[RB_MAX_K];       // its power-of-two input scaling per path
    int in, K;
};
struct Op {
    const uint32_t *bits;     // native sign tiles
    const uint16_t *g;        // fp16 [K][out]
    const uint16_t *h;        // fp16 [K][in]
    const uint16_t *x;        // fp16 [T][in]: the input buffer (read by the expansion kernel only)
    uint16_t *y;              // fp16 [T][out]
    uint8_t *up;              // expanded input of this op
    int out, in, K;
    int RT, CT;               // row tiles, column tiles
    int wg0;                  // first workgroup of this op inside its launch
    int n_cons;
    float sc[RB_MAX_K];       // power-of-two input scaling per path (max |h_k| * sc in [1/4, 1/2))
    float inv_sc[RB_MAX_K];
    Reader cons[MAX_CONS];
};

// ------------------------------------------------------------- set-up kernels ---
// PREP_SPLIT workgroups per op share the zero fill of its expanded input (padding columns and
// tokens read as zero; 1.4 MB for 11008 columns at 16 tokens); the first also works out the input
// scaling of each path, copied to the ops that read from it later by link_kernel.
constexpr int PREP_SPLIT = 8;
__global__ __launch_bounds__(256) void prep_kernel(Op *ops, int T)
{
    Op &op = ops[blockIdx.x];
    __shared__ float red[256];
    for (int p = 0; p < op.K && blockIdx.y == 0; ++p) {
        float m = 0.f;
        for (int j = threadIdx.x; j < op.in; j += 256)
            m = fmaxf(m, fabsf(__half2float(reinterpret_cast<const __half *>(op.h)[(size_t)p * op.in + j])));
        red[threadIdx.x] = m;
        __syncthreads();
        for (int s = 128; s > 0; s >>= 1) {
            if ((int)threadIdx.x < s) red[threadIdx.x] = fmaxf(red[threadIdx.x], red[threadIdx.x + s]);
            __syncthreads();
        }
        if (threadIdx.x == 0) {
            const float sc = mx::input_scale(red[0]);
            op.sc[p] = sc;
            op.inv_sc[p] = 1.f / sc;
        }
        __syncthreads();
    }
    const size_t n16 = operand_bytes(op.in, op.K, groups_of(T)) / 16;
    uint4 *up = reinterpret_cast<uint4 *>(op.up);
    for (size_t i = blockIdx.y * 256 + threadIdx.x; i < n16; i += 256 * PREP_SPLIT) up[i] = make_uint4(0, 0, 0, 0);
}

// second pass (needs every op's scaling): what a producer must know about its readers
__global__ void link_kernel(Op *ops, const int *cons_index, int n_ops)
{
    const int o = blockIdx.x * blockDim.x + threadIdx.x;
    if (o >= n_ops) return;
    Op &op = ops[o];
    for (int c = 0; c < op.n_cons; ++c) {
        const Op &m = ops[cons_index[o * MAX_CONS + c]];
        Reader r;
        r.up = m.up; r.h = m.h; r.in = m.in; r.K = m.K;
        for (int p = 0; p < RB_MAX_K; ++p) r.sc[p] = p < m.K ? m.sc[p] : 1.f;
        op.cons[c] = r;
    }
}

// Input scaling u_k = h_k (.) x (Section 4.1) for ops whose input comes from outside the stack,
// as four bf8 terms in operand order.  A thread takes 16 consecutive columns of one token and path
// (in % 32 == 0): 32 bytes of x and of h in, one 16-byte group per term out.
__global__ __launch_bounds__(256) void expand_kernel(const Op *ops, const int *which, int T)
{
    const Op &op = ops[which[blockIdx.z]];
    const int tok = blockIdx.y;
    const int nblk = op.in / 16;
    const int id = blockIdx.x * 256 + threadIdx.x;
    if (id >= nblk * op.K) return;
    const int p = id / nblk, j0 = (id - p * nblk) * 16;
    const int G = groups_of(T);
    const uint4 *xs = reinterpret_cast<const uint4 *>(reinterpret_cast<const __half *>(op.x) + (size_t)tok * op.in + j0);
    const uint4 xq[2] = {xs[0], xs[1]};
    const uint32_t xw[8] = {xq[0].x, xq[0].y, xq[0].z, xq[0].w, xq[1].x, xq[1].y, xq[1].z, xq[1].w};
    uint32_t hw[8];
    const uint16_t *hp = op.h + (size_t)p * op.in + j0;
    if (((uintptr_t)hp & 15) == 0) {                          // the scales need only be 2-byte aligned
        const uint4 h0 = reinterpret_cast<const uint4 *>(hp)[0], h1 = reinterpret_cast<const uint4 *>(hp)[1];
        hw[0] = h0.x; hw[1] = h0.y; hw[2] = h0.z; hw[3] = h0.w; hw[4] = h1.x; hw[5] = h1.y; hw[6] = h1.z; hw[7] = h1.w;
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) hw[e] = (uint32_t)hp[2 * e] | ((uint32_t)hp[2 * e + 1] << 16);
    }
    uint32_t out[4][4] = {};                                  // [term][word of the group]
    const float sc = op.sc[p];
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        const float x = __half2float(__ushort_as_half((unsigned short)(xw[e >> 1] >> (16 * (e & 1)))));
        const float h = __half2float(__ushort_as_half((unsigned short)(hw[e >> 1] >> (16 * (e & 1)))));
        const uint32_t terms = mx::expand4(h * x * sc);
#pragma unroll
        for (int t = 0; t < 4; ++t) out[t][e >> 2] |= ((terms >> (8 * t)) & 0xffu) << (8 * (e & 3));
    }
#pragma unroll
    for (int t = 0; t < 4; ++t)
        *reinterpret_cast<uint4 *>(op.up + operand_group_offset(op.K, G, j0, p, tok >> 2, 4 * (tok & 3) + t)) =
            make_uint4(out[t][0], out[t][1], out[t][2], out[t][3]);
}

// ------------------------------------------------------------------- kernel ---
// LDS ring of column tiles: a slot holds the tile's right operands and the sign tiles of the
// workgroup's row tiles; as many slots as fit (at most 16)
__host__ __device__ constexpr int slot_bytes(int K, int G, int S, int P)
{
    return (int)tile_operand_bytes(K, G) + block_tiles(S, P) * tile_words(K) * 4;
}
__host__ __device__ constexpr int ring_depth(int K, int G, int S, int P)
{
    return (144 * 1024) / slot_bytes(K, G, S, P) < 16 ? (144 * 1024) / slot_bytes(K, G, S, P) : 16;
}

// "at most rem * LPI vector-memory loads outstanding" for a run-time rem in 0 .. R.  (KERNEL only
// makes the helpers of each kernel instantiation their own.)
template <int KERNEL, int LPI, int R> struct WaitTiles {
    static __device__ __forceinline__ void run(int rem)
    {
        if (rem >= R) asm volatile("s_waitcnt vmcnt(%0)" : : "n"(R * LPI) : "memory");
        else WaitTiles<KERNEL, LPI, R - 1>::run(rem);
    }
};
template <int KERNEL, int LPI> struct WaitTiles<KERNEL, LPI, 0> {
    static __device__ __forceinline__ void run(int) { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
};

// the copies one wavefront makes per column tile: where from (advancing by `step` bytes per column
// tile), where to inside the slot, and whether the bytes are read once (sign tiles: non-temporal)
template <int KERNEL, int LPI> struct Copies {
    const uint8_t *src[LPI];
    int dst[LPI], step[LPI];
    bool once[LPI];
    __device__ __forceinline__ void request(uint8_t *slot, int ct) const
    {
#pragma unroll
        for (int i = 0; i < LPI; ++i) {
            if (once[i])
                __builtin_amdgcn_global_load_lds(src[i] + (size_t)ct * step[i], RB_LDS(slot + dst[i]), 16, 0, 2);
            else
                __builtin_amdgcn_global_load_lds(src[i] + (size_t)ct * step[i], RB_LDS(slot + dst[i]), 16, 0, 0);
        }
    }
};

template <int K, int G, int S, int P>
__global__ __launch_bounds__(THREADS, 1) void batch_kernel(const Op *__restrict__ ops, int op0, int nops, int T)
{
    constexpr int R = block_tiles(S, P), NP = 2 * K / S;     // NP: pieces per wavefront and tile
    static_assert(2 * K % S == 0 && WAVES % S == 0, "pieces and wavefronts go round");
    constexpr int OPB = (int)tile_operand_bytes(K, G);
    constexpr int TB = tile_words(K) * 4;                    // bytes of a sign tile
    constexpr int SLOT = slot_bytes(K, G, S, P);              // [operands OPB][sign tiles R x TB]
    constexpr int COPIES = SLOT / 1024;                      // 1 KB per wavefront instruction
    constexpr int LPI = (COPIES + WAVES - 1) / WAVES;        // copies per wavefront and tile
    constexpr int D = ring_depth(K, G, S, P);                 // slots in LDS; D - 1 tiles are requested ahead
    constexpr int PART = G * 4 * TILE_ROWS;                  // floats of one wavefront's partial outputs: [token][row]
    static_assert(SLOT % 1024 == 0 && D >= 2 && (D - 1) * LPI < 64, "the in-order wait counts on this");
    static_assert(WAVES * P * PART * 4 <= D * SLOT, "the partial outputs reuse the ring");
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];   // D slots

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = wave / S, sp = wave % S;
    // which op of the launch, which block of R row tiles
    int o = op0, wg = (int)blockIdx.x;
    while (o + 1 < op0 + nops && wg >= ops[o + 1].wg0) ++o;
    const Op &op = ops[o];
    wg -= op.wg0;
    const int CT = op.CT, RT = op.RT, out = op.out;
    const int rt = wg * R + r * P;                           // this wavefront's first row tile (of P)
    const bool live = rt < RT;
    const int col = lane & 15, qd = lane >> 4;
    const int scale_b = mx::term_scale(col);
    uint32_t c22;
    asm volatile("v_mov_b32 %0, 0x22222222" : "=v"(c22));

    // ---- one column tile's copies of this wavefront, always LPI of them (the waits count them):
    // the slot's bytes, 1 KB per instruction, are dealt round-robin; where the pieces do not go
    // round, a wavefront repeats a copy another one makes.  The right operands of a column tile
    // are OPB consecutive bytes; the sign tiles of the R row tiles (every one read once: non-
    // temporal) follow in the slot as they are in memory, so that lane l finds its 2 K words
    // (word c * K + k = path k, columns 128 c + 32 (l / 16) ..) at 8 K l.  A row tile past the
    // end of the matrix copies the last one (nobody reads it).
    Copies<64 * K + 8 * G + S + 128 * P, LPI> copies;
#pragma unroll
    for (int i = 0; i < LPI; ++i) {
        const int piece = (wave + WAVES * i) % COPIES;
        copies.dst[i] = piece * 1024;
        copies.once[i] = piece * 1024 >= OPB;
        if (!copies.once[i]) {
            copies.src[i] = op.up + (size_t)piece * 1024 + lane * 16;
            copies.step[i] = OPB;
        } else {
            const int b = piece * 1024 - OPB + lane * 16;
            const int rr = min(wg * R + b / TB, RT - 1);
            copies.src[i] = reinterpret_cast<const uint8_t *>(op.bits) + (size_t)rr * CT * TB + b % TB;
            copies.step[i] = TB;
        }
    }

    v4f acc[P][NP][G];
#pragma unroll
    for (int p = 0; p < P; ++p)
#pragma unroll
        for (int j = 0; j < NP; ++j)
#pragma unroll
            for (int g = 0; g < G; ++g) acc[p][j][g] = (v4f){0.f, 0.f, 0.f, 0.f};

#pragma unroll
    for (int d = 0; d < D - 1; ++d)
        if (d < CT) copies.request(lds + d * SLOT, d);
    const uint32_t lds_base = (uint32_t)(size_t)RB_LDS(lds);
    const uint32_t lds_lane = lds_base + (uint32_t)lane * 16u;
    const uint32_t lds_sign = lds_base + (uint32_t)(OPB + r * P * TB + lane * 8 * K + 4 * sp);
    int slot = 0;
    for (int ct = 0; ct < CT; ++ct) {
        // Copies complete in order and every tile costs this wavefront LPI of them: when at most
        // LPI times the number of younger tiles already requested are outstanding, tile ct is
        // here.  After the barrier it is here for every wavefront, and every wavefront is
        // through with the slot of tile ct - 1, which the next request overwrites.
        WaitTiles<64 * K + 8 * G + S + 128 * P, LPI, D - 2>::run(min(CT - 1 - ct, D - 2));
        asm volatile("s_barrier" ::: "memory");               // the barrier alone: a fence would wait for every copy in flight
        if (ct + D - 1 < CT) copies.request(lds + (slot == 0 ? D - 1 : slot - 1) * SLOT, ct + D - 1);
        if (live) {
#pragma unroll
            for (int j = 0; j < NP; ++j) {
                // Reads of the ring are written as instructions: a read the compiler can see would
                // wait for every copy still in flight.
                v8i a[P];
#pragma unroll
                for (int p = 0; p < P; ++p) {
                    uint32_t sw;
                    asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)"
                                 : "=v"(sw) : "v"(lds_sign + (uint32_t)(slot * SLOT + p * TB + 4 * j * S)) : "memory");
                    a[p][0] = (int)(((sw << 3) & 0x88888888u) | c22);
                    a[p][1] = (int)(((sw << 2) & 0x88888888u) | c22);
                    a[p][2] = (int)(((sw << 1) & 0x88888888u) | c22);
                    a[p][3] = (int)((sw & 0x88888888u) | c22);
                    a[p][4] = 0; a[p][5] = 0; a[p][6] = 0; a[p][7] = 0;
                }
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    // the operand of piece c * K + k, token group g: read once for the P row tiles
                    const uint32_t addr = lds_lane + (uint32_t)(slot * SLOT + ((sp + j * S) * G + g) * 2048);
                    v4i lo, hi;
                    asm volatile("ds_read_b128 %0, %2\n\t"
                                 "ds_read_b128 %1, %2 offset:1024\n\t"
                                 "s_waitcnt lgkmcnt(0)"
                                 : "=&v"(lo), "=&v"(hi)
                                 : "v"(addr)
                                 : "memory");
                    v8i b;
                    b[0] = lo[0]; b[1] = lo[1]; b[2] = lo[2]; b[3] = lo[3];
                    b[4] = hi[0]; b[5] = hi[1]; b[6] = hi[2]; b[7] = hi[3];
                    // A: fp4 (cbsz = 4), B: bf8 (blgp = 1); scale bytes are E8M0 exponents
#pragma unroll
                    for (int p = 0; p < P; ++p)
                        acc[p][j][g] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a[p], b, acc[p][j][g], 4, 1, 0, 0x7f7f7f7f, 0, scale_b);
                }
            }
        }
        slot = slot + 1 == D ? 0 : slot + 1;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();                                          // every wavefront is through with the operand ring

    // ---- partial outputs of this wavefront's pieces, scaled by the output scales of their paths
    // (Section 4.1: y = sum_k g_k (.) (B_k u_k)).  Lane (col, q) holds rows 4q .. 4q+3 of operand
    // column col = 4 * (token % 4) + term; the four lanes of a quad hold the four terms.
    float *const part = reinterpret_cast<float *>(lds);       // [wavefront][row tile of the wavefront][token][row]
    if (live) {
#pragma unroll
        for (int p = 0; p < P; ++p) {
            float gq[NP][4];
#pragma unroll
            for (int j = 0; j < NP; ++j) {
                const int k = (sp + j * S) % K;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int row = (rt + p) * TILE_ROWS + 4 * qd + i;
                    gq[j][i] = row < out ? (float)RB_GLOBAL(const _Float16, op.g)[(size_t)k * out + row] * op.inv_sc[k] : 0.f;
                }
            }
#pragma unroll
            for (int g = 0; g < G; ++g) {
                v4f v = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int j = 0; j < NP; ++j)
#pragma unroll
                    for (int i = 0; i < 4; ++i) v[i] = __builtin_fmaf(gq[j][i], mx::quad_sum(acc[p][j][g][i]), v[i]);
                if ((col & 3) == 0)
                    *reinterpret_cast<v4f *>(part + (wave * P + p) * PART + (4 * g + (col >> 2)) * TILE_ROWS + 4 * qd) = v;
            }
        }
    }
    __syncthreads();

    // ---- finish the R row tiles: add the S partial outputs of a row in wavefront order, round,
    // store, and write the input scaling of the ops that read y
    const int n_cons = op.n_cons;
    for (int idx = tid; idx < R * T * TILE_ROWS; idx += THREADS) {
        const int rr = idx / (T * TILE_ROWS), tok = (idx / TILE_ROWS) % T, i = idx % TILE_ROWS;
        const int row = (wg * R + rr) * TILE_ROWS + i;
        if (row >= out) continue;
        float sum = 0.f;
#pragma unroll
        for (int q = 0; q < S; ++q) sum += part[(((rr / P) * S + q) * P + rr % P) * PART + tok * TILE_ROWS + i];
        const _Float16 y16 = (_Float16)sum;                   // round to nearest even
        RB_GLOBAL(_Float16, op.y)[(size_t)tok * out + row] = y16;
        const float yf = (float)y16;
        // input scaling of the ops that read y (Section 4.1), as four bf8 terms in operand order
        for (int c = 0; c < n_cons; ++c) {
            const Reader &rd = op.cons[c];
            for (int p = 0; p < rd.K; ++p) {
                const float h = (float)RB_GLOBAL(const _Float16, rd.h)[(size_t)p * rd.in + row];
                const uint32_t terms = mx::expand4(h * yf * rd.sc[p]);
                auto *dst = RB_GLOBAL(uint8_t, rd.up) + operand_group_offset(rd.K, G, row & ~15, p, tok >> 2, 4 * (tok & 3)) + (row & 15);
#pragma unroll
                for (int t = 0; t < 4; ++t) dst[t * 16] = (uint8_t)(terms >> (8 * t));
            }
        }
    }
}

// ------------------------------------------------------------------ host ---
struct Launch { int op0, nops, groups, K, S, P; };
struct Layout { size_t ops, cons, which, up, total; };

static Layout make_layout(int n_ops, size_t up_total)
{
    Layout L;
    size_t o = 0;
    L.ops = o; o += mx::align_up(sizeof(Op) * (size_t)n_ops, 256);
    L.cons = o; o += mx::align_up(sizeof(int) * MAX_CONS * (size_t)n_ops, 256);
    L.which = o; o += mx::align_up(sizeof(int) * MAX_EXPAND, 256);
    L.up = o; o += up_total;
    L.total = mx::align_up(o, 256);
    return L;
}

bool layer_supported(const rb_layer *L, int T)
{
    return (L->K == 2 || L->K == 3) && T >= 1 && T <= MAX_T && L->in % 32 == 0;
}

size_t plan_workspace_bytes(const rb_layer *layers, int n_layers, int n_ops, int T)
{
    const int G = groups_of(T);
    size_t up_max = 0;
    for (int l = 0; l < n_layers; ++l)
        up_max = std::max(up_max, mx::align_up(operand_bytes(layers[l].in, layers[l].K, G), 256));
    return make_layout(n_ops, up_max * (size_t)n_ops).total;
}

struct Prepared {
    Layout lay;
    int n_ops = 0, T = 0, n_expand = 0, max_expand_in = 0;
    std::vector<Launch> launches;
    std::shared_ptr<std::vector<uint8_t>> blob;      // host copies of the tables: pageable, must outlive the queued copies
};
static std::mutex g_mutex;
static std::map<const void *, Prepared> g_prepared;

int prepare_plan(const rb_layer *layers, const rb_stack_op *sops, int n_ops, uint16_t *const *bufs, int T,
                 void *workspace, size_t workspace_bytes_, hipStream_t stream)
{
    if (T < 1 || T > MAX_T) return RB_ERR_UNSUPPORTED;
    const int G = groups_of(T);
    std::vector<Op> ops((size_t)n_ops);
    std::vector<int> cons((size_t)n_ops * MAX_CONS, 0), expand_list;
    std::vector<size_t> up_off((size_t)n_ops);
    size_t up_total = 0;
    for (int n = 0; n < n_ops; ++n) {
        const rb_layer &L = layers[sops[n].layer];
        if (!layer_supported(&L, T)) return RB_ERR_UNSUPPORTED;
        Op &o = ops[(size_t)n];
        std::memset(&o, 0, sizeof(Op));
        o.bits = static_cast<const uint32_t *>(L.bits);
        o.g = L.g; o.h = L.h;
        o.x = bufs[sops[n].src];
        o.y = bufs[sops[n].dst];
        o.out = L.out; o.in = L.in; o.K = L.K;
        o.RT = row_tiles(L.out); o.CT = col_tiles(L.in);
        up_off[(size_t)n] = up_total;
        up_total += mx::align_up(operand_bytes(L.in, L.K, G), 256);
        int producer = -1;
        for (int m = n - 1; m >= 0; --m)
            if (sops[m].dst == sops[n].src) { producer = m; break; }
        if (producer < 0) {
            expand_list.push_back(n);
        } else {
            Op &pr = ops[(size_t)producer];
            if (pr.n_cons >= MAX_CONS) return RB_ERR_UNSUPPORTED;
            if (pr.out != o.in) return RB_ERR_SHAPE;
            cons[(size_t)producer * MAX_CONS + pr.n_cons++] = n;
        }
    }
    if (expand_list.size() > MAX_EXPAND) return RB_ERR_UNSUPPORTED;

    // ---- launches: runs of consecutive ops of one K that neither read nor overwrite each other
    Prepared pr;
    pr.n_ops = n_ops; pr.T = T;
    for (int op0 = 0; op0 < n_ops;) {
        int nops = 0;
        const int K = ops[(size_t)op0].K;
        for (int n = op0; n < n_ops && nops < MAX_STAGE_OPS; ++n) {
            bool conflict = ops[(size_t)n].K != K;
            for (int m = op0; m < n; ++m)
                if (sops[m].dst == sops[n].src || sops[m].dst == sops[n].dst || sops[m].src == sops[n].dst) conflict = true;
            if (conflict) break;
            ++nops;
        }
        // the largest row blocks that still give the launch WANT_GROUPS workgroups, else the smallest
        Form f = form_of(K, n_forms(K) - 1);
        int groups = 0;
        for (int i = 0; i < n_forms(K); ++i) {
            f = form_of(K, i);
            groups = 0;
            for (int n = op0; n < op0 + nops; ++n) groups += (ops[(size_t)n].RT + block_tiles(f.S, f.P) - 1) / block_tiles(f.S, f.P);
            if (groups >= WANT_GROUPS) break;
        }
        groups = 0;
        for (int n = op0; n < op0 + nops; ++n) {
            ops[(size_t)n].wg0 = groups;
            groups += (ops[(size_t)n].RT + block_tiles(f.S, f.P) - 1) / block_tiles(f.S, f.P);
        }
        pr.launches.push_back(Launch{op0, nops, groups, K, f.S, f.P});
        op0 += nops;
    }
    pr.n_expand = (int)expand_list.size();
    for (int n : expand_list) pr.max_expand_in = std::max(pr.max_expand_in, ops[(size_t)n].in);
    pr.lay = make_layout(n_ops, up_total);
    const Layout &lay = pr.lay;
    if (!workspace || workspace_bytes_ < lay.total) return RB_ERR_WORKSPACE;
    uint8_t *ws = static_cast<uint8_t *>(workspace);
    for (int n = 0; n < n_ops; ++n) ops[(size_t)n].up = ws + lay.up + up_off[(size_t)n];

    pr.blob = std::make_shared<std::vector<uint8_t>>(lay.up, (uint8_t)0);
    std::vector<uint8_t> &blob = *pr.blob;
    std::memcpy(blob.data() + lay.ops, ops.data(), sizeof(Op) * (size_t)n_ops);
    std::memcpy(blob.data() + lay.cons, cons.data(), sizeof(int) * cons.size());
    if (!expand_list.empty()) std::memcpy(blob.data() + lay.which, expand_list.data(), sizeof(int) * expand_list.size());
    if (hipMemcpyAsync(ws, blob.data(), lay.up, hipMemcpyHostToDevice, stream) != hipSuccess) return RB_ERR_HIP;
    hipLaunchKernelGGL(prep_kernel, dim3(n_ops, PREP_SPLIT), dim3(256), 0, stream, reinterpret_cast<Op *>(ws + lay.ops), T);
    hipLaunchKernelGGL(link_kernel, dim3((n_ops + 63) / 64), dim3(64), 0, stream, reinterpret_cast<Op *>(ws + lay.ops),
                       reinterpret_cast<const int *>(ws + lay.cons), n_ops);
    if (hipGetLastError() != hipSuccess) return RB_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_mutex);
    g_prepared[workspace] = std::move(pr);
    return RB_OK;
}

template <int K, int G, int S, int P>
static int launch_one(const Op *d_ops, const Launch &l, int T, hipStream_t stream)
{
    const int lds_bytes = ring_depth(K, G, S, P) * slot_bytes(K, G, S, P);
    static std::atomic<bool> configured{false};
    if (!configured.load()) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(batch_kernel<K, G, S, P>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                lds_bytes) != hipSuccess)
            return RB_ERR_HIP;
        configured.store(true);
    }
    hipLaunchKernelGGL((batch_kernel<K, G, S, P>), dim3((unsigned)l.groups), dim3(THREADS), lds_bytes, stream, d_ops, l.op0, l.nops, T);
    return RB_OK;
}

template <int K, int S, int P>
static int launch_groups(const Op *d_ops, const Launch &l, int T, hipStream_t stream)
{
    switch (groups_of(T)) {
    case 1: return launch_one<K, 1, S, P>(d_ops, l, T, stream);
    case 2: return launch_one<K, 2, S, P>(d_ops, l, T, stream);
    case 3: return launch_one<K, 3, S, P>(d_ops, l, T, stream);
    default: return launch_one<K, 4, S, P>(d_ops, l, T, stream);
    }
}

// RB_ERR_UNSUPPORTED: the workspace holds no plan of this kind
int launch_plan(void *workspace, size_t workspace_bytes_, hipStream_t stream)
{
    std::unique_lock<std::mutex> lock(g_mutex);
    const auto it = g_prepared.find(workspace);
    if (it == g_prepared.end()) return RB_ERR_UNSUPPORTED;
    const Prepared &pr = it->second;
    if (workspace_bytes_ < pr.lay.total) return RB_ERR_WORKSPACE;
    uint8_t *ws = static_cast<uint8_t *>(workspace);
    const Op *d_ops = reinterpret_cast<const Op *>(ws + pr.lay.ops);
    const int T = pr.T;
    if (pr.n_expand > 0)
        hipLaunchKernelGGL(expand_kernel, dim3((pr.max_expand_in / 16 * RB_MAX_K + 255) / 256, T, (unsigned)pr.n_expand), dim3(256), 0,
                           stream, d_ops, reinterpret_cast<const int *>(ws + pr.lay.which), T);
    for (const Launch &l : pr.launches) {
        int rc = RB_ERR_UNSUPPORTED;
        if (l.K == 2) rc = l.S == 2 ? launch_groups<2, 2, 2>(d_ops, l, T, stream) : l.P == 2 ? launch_groups<2, 4, 2>(d_ops, l, T, stream)
                                    : launch_groups<2, 4, 1>(d_ops, l, T, stream);
        else if (l.K == 3) rc = launch_groups<3, 2, 1>(d_ops, l, T, stream);
        if (rc != RB_OK) return rc;
    }
    return hipGetLastError() == hipSuccess ? RB_OK : RB_ERR_HIP;
}

bool has_plan(const void *workspace)
{
    std::lock_guard<std::mutex> lock(g_mutex);
    return g_prepared.find(workspace) != g_prepared.end();
}

void forget_plan(const void *workspace)
{
    std::lock_guard<std::mutex> lock(g_mutex);
    g_prepared.erase(workspace);
}

}  // namespace batch
}  // namespace rb
