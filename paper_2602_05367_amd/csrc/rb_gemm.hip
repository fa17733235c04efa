// Many-token path of the residual-binary layer: a matrix-core GEMM.
//
// Section 4.1 / Eq. (stacked binary weight): Y[t][i] = sum_k g_k[i] * sum_j B_k[i][j] * (h_k[j] X[t][j]).
// With T in the thousands this is a dense contraction and belongs on the MFMA units:
//   * a pre-pass forms U_k = h_k (.) X once, in fp16 (input scaling, Section 4.1), times a power of
//     two s_k per path that brings max|h_k| into [1/4, 1/2): how the magnitude of a path is split
//     between g_k and h_k is not unique, and a layer that keeps it in g would otherwise push U into
//     fp16 subnormals.  The left operand carries g_k * (s_min / s_k) (a power of two at most one:
//     exact) and the result is multiplied by 1 / s_min;
//   * the GEMM contracts over the pair (path, input column) with a single accumulator: the left
//     operand element for row i is +-g_k[i] (an exact fp16 value: the stored scale with the sign
//     bit of the weight), the right operand is U_k.  Both paths land in the same fp32 sum, so
//     the path sum of Eq. (stacked binary weight) costs nothing;
//   * the left operand never exists in memory: each wavefront turns the packed sign words of its
//     rows into v_mfma_f32_32x32x16_f16 operand registers with two vector instructions per
//     register (shift so that two sign bits land on bits 15 and 31, then and-or with the packed
//     pair of |g|).  Inside a group of 32 columns the order of the contraction index is free as
//     long as both operands agree; the pre-pass stores U in the order this shift produces:
//     position 2n + hi holds the column whose sign is native bit n + 16 * hi of the word;
//   * the right operand goes through LDS, shared by the four wavefronts of a workgroup tile.  It
//     is copied global -> LDS without passing through registers, three 32-column steps ahead,
//     into a ring of four buffers with one barrier per step; rows are 64 bytes and the four
//     16-byte chunks of a row are XOR-swizzled with the token index so that neither the copy nor
//     the operand reads collide on LDS banks;
//   * the tile is 256 rows x 32 tokens (single calls of up to 32 tokens), and the contraction
//     is also split over workgroups (fp32 partial outputs in scratch, one more small kernel sums
//     and rounds them) so that a 4096-row matrix still fills the chip.  The kernel is written
//     for any split of a 256-row tile over its four wavefronts; beyond 32 tokens the
//     one-contraction kernel further down takes over, whose 256 x 256 tile shares this one's
//     staging of the right operand and its cut of the device's last round.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include <algorithm>

#include "rabit.h"
#include "rb_device.h"
#include "rb_internal.h"
#include "rb_layout.h"
#include "rb_mx_device.h"

namespace rb {
namespace gemm {

typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef unsigned v4u __attribute__((ext_vector_type(4)));

// steps between the request of a right-operand tile and its use (the ring has one buffer more): a
// step of the large tile takes about a microsecond, one of the small tile a tenth of that
constexpr int AHEAD_LARGE = 3, AHEAD_SMALL = 15;
constexpr int BLK_ROWS = 256;       // rows of a workgroup tile, both shapes
constexpr int SMALL_TOKENS = 32, LARGE_TOKENS = 256;
#define RB_LDS(p) ((__attribute__((address_space(3))) void *)(p))

// which 16-byte position of its 64-byte LDS row chunk c of a token sits at: c ^ swizzle(token)
__device__ __forceinline__ int swizzle(int token) { return ((token >> 1) ^ (token >> 3)) & 3; }

__host__ __device__ inline int round_up(int v, int a) { return (v + a - 1) / a * a; }

// position inside a group of 32 columns at which the pre-pass stores column `col` (0..31)
__host__ __device__ inline int contraction_position(int col)
{
    const int b = native_bit(col);  // bit of the native sign word
    return 2 * (b & 15) + (b >> 4);
}

// ------------------------------------------------------------- pre-pass ---
// Per call: the power-of-two input scaling of each path.  scl[k] = s_k, scl[2 + k] = s_min / s_k
// (what the left operand's |g_k| is multiplied by), scl[4] = 1 / s_min.
constexpr size_t SCALES_BYTES = 256;
__global__ __launch_bounds__(256) void hscale_kernel(const __half *__restrict__ h, int in, float *__restrict__ scl)
{
    __shared__ float red[256];
    __shared__ float sc[2];
    for (int k = 0; k < 2; ++k) {
        float m = 0.f;
        for (int j = threadIdx.x; j < in; j += 256) m = fmaxf(m, fabsf(__half2float(h[(size_t)k * in + j])));
        red[threadIdx.x] = m;
        __syncthreads();
        for (int s = 128; s > 0; s >>= 1) {
            if ((int)threadIdx.x < s) red[threadIdx.x] = fmaxf(red[threadIdx.x], red[threadIdx.x + s]);
            __syncthreads();
        }
        if (threadIdx.x == 0) sc[k] = mx::input_scale(red[0]);
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        const float s_min = fminf(sc[0], sc[1]);
        scl[0] = sc[0]; scl[1] = sc[1];
        scl[2] = s_min / sc[0]; scl[3] = s_min / sc[1];
        scl[4] = 1.f / s_min;
    }
}

// U[k][t][j'] = fp16(h_k[j] * s_k * X[t][j]); rows t >= T and columns j >= in are zero.
template <typename ActT>
__global__ __launch_bounds__(256) void scale_kernel(const ActT *__restrict__ X, const __half *__restrict__ h,
                                                    const float *__restrict__ scl, _Float16 *__restrict__ U, int T,
                                                    int T_pad, int in, int in_pad)
{
    const int j = blockIdx.x * 256 + threadIdx.x;
    const int t = blockIdx.y;
    if (j >= in_pad) return;
    const bool live = t < T && j < in;
    const float x = live ? to_float(X[(size_t)t * in + j]) : 0.f;
    const int jp = (j & ~31) + contraction_position(j & 31);
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const float hv = live ? __half2float(h[(size_t)k * in + j]) : 0.f;
        U[((size_t)k * T_pad + t) * in_pad + jp] = (_Float16)(hv * scl[k] * x);
    }
}

// split-contraction: sums the partial outputs of the `split` workgroups that share an output tile
// and rounds to the output type.  part is [split][T][rows] for rows row0 .. row0 + rows - 1 of Y.
__global__ __launch_bounds__(256) void finish_kernel(const float *__restrict__ part, const float *__restrict__ scl,
                                                     void *__restrict__ Y, int out_dtype, int T, int out, int row0,
                                                     int rows, int split, int factor)
{
    const size_t n = (size_t)T * rows;
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    float s = 0.f;
    for (int k = 0; k < split; ++k) s += part[(size_t)k * n + i];
    const size_t t = i / rows, r = i % rows;
    store_out(Y, out_dtype, t * out + row0 + r, s * scl[factor]);
}

// ----------------------------------------------------------------- GEMM ---
// "at most N vector-memory loads outstanding", then the workgroup barrier.  The immediate of
// s_waitcnt on gfx9: vmcnt in bits 3:0 and 15:14, expcnt (no wait: 7) in 6:4, lgkmcnt (no wait: 15) in 11:8.
template <int N>
__device__ __forceinline__ void wait_copies_and_sync()
{
    static_assert(N >= 0 && N < 64, "vmcnt has six bits");
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt((N & 0xf) | ((N >> 4) << 14) | (0x7 << 4) | (0xf << 8));
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// WM x WN wavefronts (four in all); a wavefront owns MP row pairs (32 rows each) x NT token tiles
// (32 tokens each).  Output tiles are numbered row block by row block.  Workgroups 0 .. full_tiles - 1
// take one tile each and all of its column tiles (those gridDim.y deals them, when the whole grid
// is split that way); the tiles after that - the last, partly filled round of the device - are
// shared by tail_split workgroups each, which take a slice of the column tiles.  Whoever covers
// only a slice writes fp32 partial sums to Acc [slice][T][tail_rows] (rows tail_row0 ..) instead
// of storing the output; finish_kernel adds the slices.
template <int OUT_DT, int WM, int WN, int MP, int NT, int AHEAD>
__global__ __launch_bounds__(256, 1) void gemm_kernel(const v4u *__restrict__ bits, const __half *__restrict__ g,
                                                      const float *__restrict__ scl, const _Float16 *__restrict__ U,
                                                      void *__restrict__ Y, float *__restrict__ Acc, int out, int RT,
                                                      int CT, int T, int T_pad,
                                                      int full_tiles, int tail_split, int tail_row0, int tail_rows)
{
    static_assert(WM * WN == 4 && WM * MP * 32 == BLK_ROWS, "tile shape");
    constexpr int BLK_TOK = WN * NT * 32;
    constexpr int NBUF = AHEAD + 1;
    constexpr int BUF_BYTES = BLK_TOK * 64;
    constexpr int GROUPS = BLK_TOK / 16;                  // copies of 16 tokens (1 KB) that fill one buffer
    constexpr int COPIES = GROUPS >= 4 ? GROUPS / 4 : 1;  // per wavefront and step (the same for all: the waits count them)
    extern __shared__ __attribute__((aligned(16))) uint8_t Bs[];       // NBUF * BUF_BYTES, given at launch

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % WM, wn = wave / WM;
    const int r = lane & 15, half_sel = (lane >> 4) & 1, kg = lane >> 5;    // row in its tile, which of two row tiles, k group
    const int in_pad = CT * TILE_COLS;
    // workgroups that share a token block sit on the same XCD (ids are dealt round-robin over
    // eight of them), so the slice of U they all walk stays in that XCD's L2
    const int TB = T_pad / BLK_TOK;
    int tile = (int)blockIdx.x, slice = (int)blockIdx.y, n_slices = (int)gridDim.y;
    if (tile >= full_tiles) {
        const int u = tile - full_tiles;
        tile = full_tiles + u / tail_split;
        slice = u % tail_split;
        n_slices = tail_split;
    }
    const bool partial = n_slices > 1;
    const int tb = tile % TB, rb = tile / TB;
    const int rt_base = rb * (BLK_ROWS / TILE_ROWS) + wm * MP * 2;           // first row tile of this wavefront
    // column tiles of this workgroup
    const int ct_begin = (int)((long)CT * slice / n_slices);
    const int ct_end = (int)((long)CT * (slice + 1) / n_slices);

    // ---- per-row constants: |g| as a packed pair, and whether the sign bits must be flipped
    // flip[i]: for the row this lane holds sign words of (row tile i, row r); G2[m]: for the row this
    // lane feeds to the matrix instruction (row pair m, row l % 32)
    uint32_t G2[MP][2], flip[2 * MP][2];
#pragma unroll
    for (int i = 0; i < 2 * MP; ++i) {
        const int row = (rt_base + i) * TILE_ROWS + r;
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            const uint32_t gb = row < out ? (uint32_t)__half_as_ushort(g[(size_t)k * out + row]) : 0u;
            flip[i][k] = (gb & 0x8000u) ? 0xffffffffu : 0u;
        }
    }
#pragma unroll
    for (int m = 0; m < MP; ++m) {
        const int row = (rt_base + 2 * m + half_sel) * TILE_ROWS + r;
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            // |g| times s_min / s_k: a power of two at most one, exact short of fp16 underflow
            const float gv = row < out ? fabsf(__half2float(g[(size_t)k * out + row])) * scl[2 + k] : 0.f;
            const uint32_t mag = (uint32_t)__half_as_ushort(__float2half_rn(gv));
            G2[m][k] = mag | (mag << 16);
        }
    }
    // A 32 x 32 x 16 instruction covers half a step: lane (row l % 32, k group kg = l / 32) of half
    // kk holds positions 16kk + 8kg .. +7: register e gets native bits n and n + 16, n = 8kk + 4kg + e,
    // on bits 15 and 31
    uint32_t sh[2][4];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
#pragma unroll
        for (int e = 0; e < 4; ++e) sh[kk][e] = (uint32_t)(15 - 8 * kk - 4 * kg - e);

    // sign words of this wavefront's row tiles for one column tile: lane (r, q) holds, for row r,
    // the four words [column half c][path k] of columns 128c + 32q .. +31
    auto load_words = [&](int ct, v4u (&w)[2 * MP]) {
#pragma unroll
        for (int i = 0; i < 2 * MP; ++i) {
            const int rt = rt_base + i;
            v4u v = {0u, 0u, 0u, 0u};
            if (rt < RT) v = bits[((size_t)rt * CT + ct) * 64 + lane];
            v[0] ^= flip[i][0]; v[1] ^= flip[i][1]; v[2] ^= flip[i][0]; v[3] ^= flip[i][1];
            w[i] = v;
        }
    };
    // one of the four words again, for the next column tile, once its last use is behind
    auto reload_word = [&](int ct, int comp, v4u (&w)[2 * MP]) {
        const uint32_t *words = reinterpret_cast<const uint32_t *>(bits);
#pragma unroll
        for (int i = 0; i < 2 * MP; ++i) {
            const int rt = rt_base + i;
            uint32_t v = 0u;
            if (rt < RT) v = words[(((size_t)rt * CT + ct) * 64 + lane) * 4 + comp];
            w[i][comp] = v ^ flip[i][comp & 1];
        }
    };

    // right-operand staging: one copy instruction moves 16 tokens x 64 bytes; lane L lands at LDS
    // position (token L / 4, chunk position L % 4) and therefore fetches chunk
    // (L % 4) ^ swizzle(token) from memory.  With fewer than four groups some wavefronts repeat a
    // copy another one makes (same bytes to the same place).
    const uint8_t *stage_src[COPIES];
    int stage_group[COPIES];
#pragma unroll
    for (int j = 0; j < COPIES; ++j) {
        stage_group[j] = (wave * COPIES + j) % GROUPS;
        const int token = 16 * stage_group[j] + (lane >> 2);
        const int chunk = (lane & 3) ^ swizzle(token);
        stage_src[j] = reinterpret_cast<const uint8_t *>(U + ((size_t)tb * BLK_TOK + token) * in_pad + chunk * 8);
    }
    const size_t path_stride = (size_t)T_pad * in_pad * sizeof(_Float16);
    // step s = 16 (ct - ct_begin) + (8 path + 4 column half + 32-column group); its right operand
    // lives in buffer s % NBUF
    const int n_steps = (ct_end - ct_begin) * 16;
    auto stage_step = [&](int s) {
        // past the end: repeat the first copy, so that the number of copies per step stays constant
        const int sc = s < n_steps ? s : 0;
        const size_t off = ((sc >> 3) & 1) * path_stride +
                           (size_t)((ct_begin + (sc >> 4)) * TILE_COLS + (sc & 7) * 32) * sizeof(_Float16);
#pragma unroll
        for (int j = 0; j < COPIES; ++j)
            __builtin_amdgcn_global_load_lds(static_cast<const void *>(stage_src[j] + off),
                                             RB_LDS(&Bs[(s % NBUF) * BUF_BYTES + stage_group[j] * 1024]), 16, 0, 0);
    };
    // operand reads are written as instructions: a read the compiler can see would make it wait for
    // every copy still in flight
    uint32_t b_addr[NT][2];
#pragma unroll
    for (int n = 0; n < NT; ++n) {
        const int token = (wn * NT + n) * 32 + (lane & 31);
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
            b_addr[n][kk] = (uint32_t)(size_t)RB_LDS(&Bs[token * 64 + (((2 * kk + kg) ^ swizzle(token)) * 16)]);
    }

    v16f acc[MP][NT];
#pragma unroll
    for (int m = 0; m < MP; ++m)
#pragma unroll
        for (int n = 0; n < NT; ++n)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[m][n][e] = 0.f;

    v4u cur[2 * MP];
    v8h a[2][MP][2], b[2][NT][2];
    uint32_t wq[MP], wsel0[MP], wsel1[MP];
    const uint32_t sel_mask = half_sel ? 0xffffffffu : 0u;      // which of the two fetched words is this lane's
    // the pieces of work one step does for the next one, so that they can be spread between the
    // matrix instructions: B reads (NT * 2), word fetches (MP), register expansions (MP * 4 pairs)
    auto read_b = [&](int s, int i, v8h (&bb)[NT][2]) {
        asm volatile("ds_read_b128 %0, %1" : "=v"(bb[i >> 1][i & 1])
                     : "v"(b_addr[i >> 1][i & 1] + (uint32_t)((s % NBUF) * BUF_BYTES)) : "memory");
    };
    auto fetch_a = [&](const v4u (&w)[2 * MP], int k, int c, int q, int m) {
        // every lane gets the word of its row (row tile 2m + half_sel, row r) from lane (r, q) of
        // that tile's register
        wsel0[m] = (uint32_t)__shfl((int)w[2 * m][c * 2 + k], r + 16 * q);
        wsel1[m] = (uint32_t)__shfl((int)w[2 * m + 1][c * 2 + k], r + 16 * q);
    };
    auto expand_a = [&](int i, int k, v8h (&aa)[MP][2]) {
        // two of the four registers of (row pair m, half kk)
        const int m = i >> 2, kk = (i >> 1) & 1, e0 = (i & 1) * 2;
        if ((i & 3) == 0) wq[m] = (wsel0[m] & ~sel_mask) | (wsel1[m] & sel_mask);     // one bit-field insert
        union { v8h h; uint32_t u[4]; } f;
        f.h = aa[m][kk];
#pragma unroll
        for (int e = e0; e < e0 + 2; ++e) f.u[e] = ((wq[m] << sh[kk][e]) & 0x80008000u) | G2[m][k];
        aa[m][kk] = f.h;
    };
    auto wait_b = [&](v8h (&bb)[NT][2]) {
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
        for (int n = 0; n < NT; ++n) asm volatile("" : "+v"(bb[n][0]), "+v"(bb[n][1]));
    };

    if (n_steps > 0) {
        // ---- prologue: NBUF steps of copies in flight, operands of step 0 in registers
        load_words(ct_begin, cur);
#pragma unroll
        for (int s = 0; s < NBUF; ++s) stage_step(s);
#pragma unroll
        for (int m = 0; m < MP; ++m) fetch_a(cur, 0, 0, 0, m);
#pragma unroll
        for (int i = 0; i < MP * 4; ++i) expand_a(i, 0, a[0]);
        wait_copies_and_sync<COPIES * AHEAD>();
#pragma unroll
        for (int i = 0; i < NT * 2; ++i) read_b(0, i, b[0]);
        wait_b(b[0]);
    }

    // ---- main loop.  One wavefront runs per SIMD, so nothing but its own instruction order keeps
    // the matrix pipe busy: the matrix instructions of step s are interleaved with everything step
    // s + 1 needs (barrier, copy request, operand reads, sign expansion).
    constexpr int SLOTS = MP * NT * 2;                          // matrix instructions per step
    constexpr int JOBS = 2 + NT * 2 + MP + MP * 4;              // sync, copies, B reads, fetches, expansions
    for (int ct = ct_begin; ct < ct_end; ++ct) {
#pragma unroll
        for (int step = 0; step < 16; ++step) {
            const int s = (ct - ct_begin) * 16 + step;
            const int p = step & 1, pn = p ^ 1;                       // register sets of this step and the next
            const int ns = (step + 1) & 15;                           // next step inside its column tile
            const int k_ = ns >> 3, c_ = (ns >> 2) & 1, q_ = ns & 3;
#pragma unroll
            for (int j = 0; j < SLOTS; ++j) {
                const int kk = j / (MP * NT), n = (j / MP) % NT, m = j % MP;
                acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[p][m][kk], b[p][n][kk], acc[m][n], 0, 0, 0);
#pragma unroll
                for (int job = j * JOBS / SLOTS; job < (j + 1) * JOBS / SLOTS; ++job) {
                    if (job == 0) {
                        // The copies of step s + 1 were requested AHEAD steps before that step and
                        // COPIES * (AHEAD - 1) copies came after them (the sign-word loads at the top of
                        // a column tile only make this wait longer than needed).  Every wavefront has
                        // read its operands of step s before it gets here, so after the barrier the
                        // buffer of step s may be overwritten.
                        wait_copies_and_sync<COPIES * (AHEAD - 1)>();
                    } else if (job == 1) {
                        stage_step(s + NBUF);
                    } else if (job < 2 + NT * 2) {
                        read_b(s + 1, job - 2, b[pn]);
                    } else if (job < 2 + NT * 2 + MP) {
                        fetch_a(cur, k_, c_, q_, job - (2 + NT * 2));
                    } else {
                        expand_a(job - (2 + NT * 2 + MP), k_, a[pn]);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            wait_b(b[pn]);
            // The four steps that use word [c][k] end with step 8k + 4c + 3, and the fetch for that
            // step happened one step earlier: the register is free for the next column tile, which
            // needs it 13 steps from now at the earliest.
            if ((step & 3) == 3 && ct + 1 < ct_end) reload_word(ct + 1, ((step >> 2) & 1) * 2 + (step >> 3), cur);
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // no copy may land in LDS after the end

    // ---- epilogue: lane l of tile (m, n) holds token 32n + l % 32 and, in register 4a + e, row
    // 8a + 4 (l / 32) + e of the 32.  (The width is passed through an opaque statement so that
    // none of the address arithmetic below is computed ahead of the main loop, where registers
    // are scarce.)
    asm volatile("" : "+s"(out));
    const float inv_s = scl[4];
#pragma unroll
    for (int n = 0; n < NT; ++n) {
        const int t = tb * BLK_TOK + (wn * NT + n) * 32 + (lane & 31);
        if (t >= T) continue;
#pragma unroll
        for (int m = 0; m < MP; ++m) {
#pragma unroll
            for (int a4 = 0; a4 < 4; ++a4) {
                const int row0 = (rt_base + 2 * m) * TILE_ROWS + 8 * a4 + 4 * kg;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (row0 + e >= out) continue;
                    if (partial)
                        Acc[((size_t)slice * T + t) * tail_rows + (row0 + e - tail_row0)] = acc[m][n][4 * a4 + e];
                    else
                        store_out(Y, OUT_DT, (size_t)t * out + row0 + e, acc[m][n][4 * a4 + e] * inv_s);
                }
            }
        }
    }
}

// ------------------------------------------------- one contraction (prefill) ---
// With hundreds of tokens per weight the dense form of the layer, Y = W_hat X with
// W_hat = sum_k g_k (.) B_k (.) h_k (Alg. 2, "compute layer output"), needs half the matrix
// instructions of the two contractions above: the left operand is the effective weight itself,
// built in registers from the packed signs on the way to the matrix instruction and never stored.
// Per pair of fp16 elements: |g_1| |h_1| (packed multiply), its sign from the sign word (shift,
// and-or), the signed |h_2| (shift, and-or), and one packed fused multiply-add with |g_2|: six
// vector instructions, two roundings to fp16 (the product of path 1 and the sum).  Signs of g are
// folded into the sign words per row, signs of h per 32-column group (a word the pre-pass writes),
// so the magnitudes are non-negative and the and-or can place the sign.  Magnitudes are scaled by
// powers of two (h_k by s_k as above, g_k by S / s_k with one S for both paths) so that the
// products sit in fp16's normal range however the layer splits its magnitude; the result is
// multiplied by 1 / S.  The right operand is X itself in fp16, in the contraction order of the
// sign words.  A workgroup tile is 256 rows x 256 tokens; each of the four wavefronts owns 64 rows
// and all 256 tokens, so no two wavefronts build the same left operand.
constexpr int ONE_NBUF = 5;                    // ring of right-operand buffers (three steps of copies in flight)
constexpr int ONE_BUF_BYTES = LARGE_TOKENS * 64 + 256;     // 256 tokens x 32 columns of X, then the step's h block
constexpr int HBLOCK_BYTES = 256;              // per 32-column group: [path][32 magnitudes fp16][K sign words][padding]

// Largest |h_k| and |g_k|: ABSMAX_GROUPS workgroups take a slice each and write their four maxima
// to part[group][4] (scratch that the next kernels overwrite)
constexpr int ABSMAX_GROUPS = 64;
// (part[group][2 k] for |h_k|, part[group][2 k + 1] for |g_k|, eight floats per group)
__global__ __launch_bounds__(256) void absmax_kernel(const __half *__restrict__ g, const __half *__restrict__ h, int K, int out,
                                                     int in, float *__restrict__ part)
{
    __shared__ float red[2 * RB_MAX_K][256];
    float m[2 * RB_MAX_K];
#pragma unroll
    for (int q = 0; q < 2 * RB_MAX_K; ++q) m[q] = 0.f;
    const int tid = blockIdx.x * 256 + threadIdx.x, stride = ABSMAX_GROUPS * 256;
#pragma unroll
    for (int k = 0; k < RB_MAX_K; ++k) {
        if (k < K) {
            for (int j = tid; j < in; j += stride) m[2 * k] = fmaxf(m[2 * k], fabsf(__half2float(h[(size_t)k * in + j])));
            for (int j = tid; j < out; j += stride) m[2 * k + 1] = fmaxf(m[2 * k + 1], fabsf(__half2float(g[(size_t)k * out + j])));
        }
    }
#pragma unroll
    for (int q = 0; q < 2 * RB_MAX_K; ++q) red[q][threadIdx.x] = m[q];
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s)
#pragma unroll
            for (int q = 0; q < 2 * RB_MAX_K; ++q) red[q][threadIdx.x] = fmaxf(red[q][threadIdx.x], red[q][threadIdx.x + s]);
        __syncthreads();
    }
    if (threadIdx.x < 2 * RB_MAX_K) part[blockIdx.x * 8 + threadIdx.x] = red[threadIdx.x][0];
}

// scl[k] = s_k (h), scl[3 + k] = S / s_k (g), scl[6] = 1 / S, with S the largest common power of two
// that keeps every path's |g_k| S / s_k at or below 1/2
__global__ __launch_bounds__(64) void scales1_kernel(const float *__restrict__ part, int K, float *__restrict__ scl)
{
    float m[2 * RB_MAX_K];
#pragma unroll
    for (int q = 0; q < 2 * RB_MAX_K; ++q) {
        m[q] = part[threadIdx.x * 8 + q];                   // ABSMAX_GROUPS = 64 = one per lane
        for (int s = 32; s > 0; s >>= 1) m[q] = fmaxf(m[q], __shfl_xor(m[q], s));
    }
    if (threadIdx.x == 0) {
        float sk[RB_MAX_K], S = 0.f;
        for (int k = 0; k < K; ++k) {
            sk[k] = mx::input_scale(m[2 * k]);
            const float cand = sk[k] * mx::input_scale(m[2 * k + 1]);
            S = k == 0 ? cand : fminf(S, cand);
        }
        for (int k = 0; k < K; ++k) { scl[k] = sk[k]; scl[3 + k] = S / sk[k]; }
        scl[6] = 1.f / S;
    }
}

// the h block of every 32-column group, and X in fp16 in contraction order (rows t >= T and columns
// j >= in are zero)
__global__ __launch_bounds__(32 * RB_MAX_K) void hblock_kernel(const __half *__restrict__ h, const float *__restrict__ scl, int K,
                                                               int in, uint8_t *__restrict__ Hblk)
{
    // one thread per (path, column) of the group: threads 0..31 path 0, 32..63 path 1, 64..95 path 2
    const int group = blockIdx.x, k = threadIdx.x >> 5, col = threadIdx.x & 31;
    uint8_t *blk = Hblk + (size_t)group * HBLOCK_BYTES;
    if (k >= K) {
        // the rest of the block: nobody reads it, but it is copied
        for (int i = K * 64 + K * 4 + 4 * col; i < HBLOCK_BYTES; i += 128) *reinterpret_cast<uint32_t *>(blk + i) = 0u;
        return;
    }
    const int j = group * 32 + col;
    const float hv = j < in ? __half2float(h[(size_t)k * in + j]) : 0.f;
    reinterpret_cast<_Float16 *>(blk)[k * 32 + contraction_position(col)] = (_Float16)(fabsf(hv) * scl[k]);
    // sign word in the bit order of the stored sign words: native bit of column col
    const unsigned long long neg = __ballot(hv < 0.f);       // a wavefront holds two paths (or path 2 alone)
    const uint32_t mine = (uint32_t)(neg >> (32 * (threadIdx.x >> 5 & 1)));
    uint32_t word = 0;
    for (int b = 0; b < 32; ++b) word |= ((mine >> b) & 1u) << native_bit(b);
    if (col == 0) reinterpret_cast<uint32_t *>(blk + K * 64)[k] = word;
    if (K == RB_MAX_K && k == 0)
        for (int i = K * 64 + K * 4 + 4 * col; i < HBLOCK_BYTES; i += 128) *reinterpret_cast<uint32_t *>(blk + i) = 0u;
}

// a thread writes eight consecutive positions (16 bytes) of a 32-column group and gathers their
// eight columns from the group's 64 bytes of X
template <typename ActT>
__global__ __launch_bounds__(256) void xperm_kernel(const ActT *__restrict__ X, _Float16 *__restrict__ Xp, int T, int T_pad,
                                                    int in, int in_pad)
{
    const int p8 = blockIdx.x * 256 + threadIdx.x;          // which run of eight positions of the row
    const int t = blockIdx.y;
    if (p8 * 8 >= in_pad) return;
    const int group = p8 >> 2, pos0 = (p8 & 3) * 8;
    v8h o;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        // position 2n + hi holds the column of native bit n + 16 hi
        const int pos = pos0 + e, bit = (pos >> 1) + 16 * (pos & 1);
        const int j = group * 32 + column_of_native_bit(bit);
        o[e] = (_Float16)((t < T && j < in) ? to_float(X[(size_t)t * in + j]) : 0.f);
    }
    *reinterpret_cast<v8h *>(Xp + (size_t)t * in_pad + (size_t)p8 * 8) = o;
}

typedef _Float16 v2h __attribute__((ext_vector_type(2)));

template <int OUT_DT, int K>
__global__ __launch_bounds__(256, 1) void gemm1_kernel(const uint32_t *__restrict__ bits, const __half *__restrict__ g,
                                                       const float *__restrict__ scl, const uint8_t *__restrict__ Hblk,
                                                       const _Float16 *__restrict__ Xp, void *__restrict__ Y,
                                                       float *__restrict__ Acc, int out, int RT, int CT, int T, int T_pad,
                                                       int full_tiles, int tail_split, int tail_row0, int tail_rows)
{
    constexpr int MP = 2, NT = 8, BLK_TOK = LARGE_TOKENS, NBUF = ONE_NBUF, BUF_BYTES = ONE_BUF_BYTES;
    constexpr int COPIES = 4;                              // 16 groups of 16 tokens over four wavefronts
    constexpr int CP = COPIES + 1;                         // copies per wavefront and step: X, and the h block
    extern __shared__ __attribute__((aligned(16))) uint8_t Bs[];       // NBUF * BUF_BYTES

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 15, half_sel = (lane >> 4) & 1, kg = lane >> 5;
    const int in_pad = CT * TILE_COLS;
    const int TB = T_pad / BLK_TOK;
    int tile = (int)blockIdx.x, slice = 0, n_slices = 1;
    if (tile >= full_tiles) {
        const int u = tile - full_tiles;
        tile = full_tiles + u / tail_split;
        slice = u % tail_split;
        n_slices = tail_split;
    }
    const bool partial = n_slices > 1;
    const int tb = tile % TB, rb = tile / TB;
    const int rt_base = rb * (BLK_ROWS / TILE_ROWS) + wave * MP * 2;           // first row tile of this wavefront
    const int ct_begin = (int)((long)CT * slice / n_slices);
    const int ct_end = (int)((long)CT * (slice + 1) / n_slices);

    // ---- per-row constants: |g_k| S / s_k as a packed pair, and the sign of g_k as a mask on the sign words
    // (both for the row this lane feeds to the matrix instruction: row pair m, row l % 32)
    uint32_t G2[MP][K], flip[MP][K];
#pragma unroll
    for (int m = 0; m < MP; ++m) {
        const int row = (rt_base + 2 * m + half_sel) * TILE_ROWS + r;
#pragma unroll
        for (int k = 0; k < K; ++k) {
            const __half gk = row < out ? g[(size_t)k * out + row] : __float2half(0.f);
            flip[m][k] = (__half_as_ushort(gk) & 0x8000u) ? 0xffffffffu : 0u;
            const float gv = fabsf(__half2float(gk)) * scl[3 + k];
            const uint32_t mag = (uint32_t)__half_as_ushort(__float2half_rn(gv));
            G2[m][k] = mag | (mag << 16);
        }
    }
    // lane (row, k group kg) holds positions 16 kk + 8 kg .. + 7: register e of half kk gets native
    // bits n and n + 16, n = 8 kk + 4 kg + e, on bits 15 and 31.  The words are shifted right by
    // 4 kg once per step; what is left of the shift is a constant.
    const uint32_t kg4 = 4u * (uint32_t)kg;

    // sign words of this wavefront's row tiles for one column tile: lane (r, q) holds, for row r,
    // the 2 K words [column half c][path k] of columns 128c + 32q .. +31
    struct Words { uint32_t w[2 * K]; };
    auto load_half = [&](int ct, int c, Words (&w)[2 * MP]) {
#pragma unroll
        for (int i = 0; i < 2 * MP; ++i) {
            const int rt = rt_base + i;
            const uint32_t *src = bits + (((size_t)rt * CT + ct) * 64 + lane) * (2 * K) + c * K;
#pragma unroll
            for (int k = 0; k < K; ++k) w[i].w[c * K + k] = rt < RT ? src[k] : 0u;
        }
    };
    auto load_words = [&](int ct, Words (&w)[2 * MP]) {
        load_half(ct, 0, w);
        load_half(ct, 1, w);
    };
    // the words of column half c again, for the next column tile
    auto reload_half = [&](int ct, int c, Words (&w)[2 * MP]) { load_half(ct, c, w); };

    // right-operand staging, as in the kernel above, plus the 256-byte h block of the step (every
    // wavefront copies it: four bytes per lane, the same bytes to the same place)
    // (a base the wavefront shares plus a 32-bit offset per lane: a token block of X is < 4 GB)
    const uint8_t *stage_base = reinterpret_cast<const uint8_t *>(Xp + (size_t)tb * BLK_TOK * in_pad);
    uint32_t stage_off[COPIES];
#pragma unroll
    for (int j = 0; j < COPIES; ++j) {
        const int token = 16 * (wave * COPIES + j) + (lane >> 2);
        const int chunk = (lane & 3) ^ swizzle(token);
        stage_off[j] = (uint32_t)(((size_t)token * in_pad + chunk * 8) * sizeof(_Float16));
    }
    // step s = 8 (ct - ct_begin) + 4 column half + 32-column group; its operands live in buffer s % NBUF
    const int n_steps = (ct_end - ct_begin) * 8;
    auto stage_step = [&](int s) {
        const int sc = s < n_steps ? s : 0;               // past the end: repeat the first copy
        const int group = ct_begin * 8 + sc;              // 32-column group of the matrix
        uint8_t *buf = &Bs[(s % NBUF) * BUF_BYTES];
        const uint8_t *src = stage_base + (size_t)group * 64;
#pragma unroll
        for (int j = 0; j < COPIES; ++j)
            __builtin_amdgcn_global_load_lds(static_cast<const void *>(src + stage_off[j]),
                                             RB_LDS(buf + (wave * COPIES + j) * 1024), 16, 0, 0);
        __builtin_amdgcn_global_load_lds(static_cast<const void *>(Hblk + (size_t)group * HBLOCK_BYTES + lane * 4),
                                         RB_LDS(buf + LARGE_TOKENS * 64), 4, 0, 0);
    };
    // LDS addresses of this lane's operand reads inside a buffer: token tile n adds n * 2048
    uint32_t b_addr[2];
    {
        const int token = lane & 31;
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) b_addr[kk] = (uint32_t)(size_t)RB_LDS(&Bs[token * 64 + (((2 * kk + kg) ^ swizzle(token)) * 16)]);
    }
    const uint32_t h_addr = (uint32_t)(size_t)RB_LDS(&Bs[LARGE_TOKENS * 64 + 16 * kg]);

    v16f acc[MP][NT];
#pragma unroll
    for (int m = 0; m < MP; ++m)
#pragma unroll
        for (int n = 0; n < NT; ++n)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[m][n][e] = 0.f;

    Words cur[2 * MP];
    v8h a[2][MP][2], b[NT][2];
    v8h hm[K][2];                                             // [path][half]: |h| of this lane's eight positions
    uint32_t hs[K];                                           // sign words of h for the step
    uint32_t wq[MP][K];
    const uint32_t sel_mask = half_sel ? 0xffffffffu : 0u;
    // (addresses: one register per half and ring buffer, everything else in the instruction's offset)
    auto read_b = [&](uint32_t addr, int n, int kk) {
        switch (n) {
        case 0: asm volatile("ds_read_b128 %0, %1" : "=v"(b[0][kk]) : "v"(addr) : "memory"); break;
        case 1: asm volatile("ds_read_b128 %0, %1 offset:2048" : "=v"(b[1][kk]) : "v"(addr) : "memory"); break;
        case 2: asm volatile("ds_read_b128 %0, %1 offset:4096" : "=v"(b[2][kk]) : "v"(addr) : "memory"); break;
        case 3: asm volatile("ds_read_b128 %0, %1 offset:6144" : "=v"(b[3][kk]) : "v"(addr) : "memory"); break;
        case 4: asm volatile("ds_read_b128 %0, %1 offset:8192" : "=v"(b[4][kk]) : "v"(addr) : "memory"); break;
        case 5: asm volatile("ds_read_b128 %0, %1 offset:10240" : "=v"(b[5][kk]) : "v"(addr) : "memory"); break;
        case 6: asm volatile("ds_read_b128 %0, %1 offset:12288" : "=v"(b[6][kk]) : "v"(addr) : "memory"); break;
        default: asm volatile("ds_read_b128 %0, %1 offset:14336" : "=v"(b[7][kk]) : "v"(addr) : "memory"); break;
        }
    };
    // addr: this lane's 16 bytes of path 0, half 0 of the step's h block; reads 0 .. 2K - 1 are the
    // magnitudes [path][half], read 2K the sign words (K * 64 bytes into the block; addr carries
    // 16 bytes per k group)
    auto read_h = [&](uint32_t addr, int i) {
        switch (i) {
        case 0: asm volatile("ds_read_b128 %0, %1" : "=v"(hm[0][0]) : "v"(addr) : "memory"); break;
        case 1: asm volatile("ds_read_b128 %0, %1 offset:32" : "=v"(hm[0][1]) : "v"(addr) : "memory"); break;
        case 2: asm volatile("ds_read_b128 %0, %1 offset:64" : "=v"(hm[1][0]) : "v"(addr) : "memory"); break;
        case 3: asm volatile("ds_read_b128 %0, %1 offset:96" : "=v"(hm[1][1]) : "v"(addr) : "memory"); break;
        default:
            if constexpr (K == 3) {
                if (i == 4) { asm volatile("ds_read_b128 %0, %1 offset:128" : "=v"(hm[K - 1][0]) : "v"(addr) : "memory"); break; }
                if (i == 5) { asm volatile("ds_read_b128 %0, %1 offset:160" : "=v"(hm[K - 1][1]) : "v"(addr) : "memory"); break; }
                v4u v;
                asm volatile("ds_read_b128 %0, %1 offset:192" : "=v"(v) : "v"(addr - 16u * (uint32_t)kg) : "memory");
                hs[0] = v[0]; hs[1] = v[1]; hs[K - 1] = v[2];
            } else {
                uint2 v;
                asm volatile("ds_read_b64 %0, %1 offset:128" : "=v"(v) : "v"(addr - 16u * (uint32_t)kg) : "memory");
                hs[0] = v.x; hs[1] = v.y;
            }
            break;
        }
    };
    auto ring = [&](int s) { return (uint32_t)((s % NBUF) * BUF_BYTES); };
    // The word of this lane's row (row tile 2m + half_sel, row r) sits in lane (r, q) of that
    // tile's register.  The lane exchange is written as instructions, like the operand reads: its
    // results are taken up after the step's common wait, not one by one.
    uint32_t wf[MP][K][2];
    const uint32_t bp_addr = 4u * (uint32_t)r;
    auto fetch_a = [&](const Words (&w)[2 * MP], int c, int q, int m, int k) {
        const uint32_t a0 = bp_addr + 64u * (uint32_t)q;
        asm volatile("ds_bpermute_b32 %0, %1, %2" : "=v"(wf[m][k][0]) : "v"(a0), "v"(w[2 * m].w[c * K + k]) : "memory");
        asm volatile("ds_bpermute_b32 %0, %1, %2" : "=v"(wf[m][k][1]) : "v"(a0), "v"(w[2 * m + 1].w[c * K + k]) : "memory");
    };
    // after the wait: pick the word of this lane's row tile, put the signs of g and h into it, and
    // move it so that this lane's first position sits at bit 0 (and 16)
    auto sign_a = [&](int m, int k) {
        asm volatile("" : "+v"(wf[m][k][0]), "+v"(wf[m][k][1]));
        const uint32_t w = (wf[m][k][0] & ~sel_mask) | (wf[m][k][1] & sel_mask);
        wq[m][k] = (w ^ hs[k] ^ flip[m][k]) >> kg4;
    };
    auto expand_a = [&](int i, v8h (&aa)[MP][2]) {
        // register e of the four of (row pair m, half kk): two elements of the effective weight
        const int m = i >> 3, kk = (i >> 2) & 1, e = i & 3;
        union { v8h h; uint32_t u[4]; v2h p[4]; } f, h0;
        f.h = aa[m][kk];
        h0.h = hm[0][kk];
        union { uint32_t u; v2h p; } g0, p1;
        g0.u = G2[m][0];
        p1.p = g0.p * h0.p[e];                                                 // |g_1| |h_1|
        p1.u = ((wq[m][0] << (15 - 8 * kk - e)) & 0x80008000u) | p1.u;          // its sign
#pragma unroll
        for (int k = 1; k < K; ++k) {
            union { v8h h; uint32_t u[4]; } hk;
            union { uint32_t u; v2h p; } gk, sk;
            hk.h = hm[k][kk];
            gk.u = G2[m][k];
            sk.u = ((wq[m][k] << (15 - 8 * kk - e)) & 0x80008000u) | hk.u[e];   // signed |h_k|
            p1.p = __builtin_elementwise_fma(gk.p, sk.p, p1.p);
        }
        f.p[e] = p1.p;
        aa[m][kk] = f.h;
    };
    auto wait_lds = [&]() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); };
    auto touch_h = [&]() {
#pragma unroll
        for (int k = 0; k < K; ++k) asm volatile("" : "+v"(hm[k][0]), "+v"(hm[k][1]), "+v"(hs[k]));
    };
    auto touch_b = [&](int kk) {
#pragma unroll
        for (int n = 0; n < NT; ++n) asm volatile("" : "+v"(b[n][kk]));
    };

    if (n_steps > 0) {
        // ---- prologue: NBUF - 1 steps of copies in flight; operands of step 0 in registers
        load_words(ct_begin, cur);
#pragma unroll
        for (int s = 0; s < NBUF - 1; ++s) stage_step(s);
        wait_copies_and_sync<CP * (NBUF - 2)>();               // step 0 has landed
#pragma unroll
        for (int i = 0; i < 2 * K + 1; ++i) read_h(h_addr, i);
#pragma unroll
        for (int m = 0; m < MP; ++m)
#pragma unroll
            for (int k = 0; k < K; ++k) fetch_a(cur, 0, 0, m, k);
#pragma unroll
        for (int n = 0; n < NT; ++n) read_b(b_addr[0], n, 0);
        wait_lds();
        touch_h();
        touch_b(0);
#pragma unroll
        for (int m = 0; m < MP; ++m)
#pragma unroll
            for (int k = 0; k < K; ++k) sign_a(m, k);
#pragma unroll
        for (int i = 0; i < MP * 8; ++i) expand_a(i, a[0]);
    }

    // ---- main loop: 32 matrix instructions per step (2 row pairs x 8 token tiles x 2 halves).  In
    // between: the second half of this step's right operand (slots 0-7), everything the next
    // step's left operand needs (h block, sign words, expansion) and the first half of its right
    // operand (slots 16-23, after that half's last use).
    for (int ct = ct_begin; ct < ct_end; ++ct) {
#pragma unroll
        for (int step = 0; step < 8; ++step) {
            const int s = (ct - ct_begin) * 8 + step;
            const int p = step & 1, pn = p ^ 1;
            const int ns = (step + 1) & 7;
            const int c_ = ns >> 2, q_ = ns & 3;
            const uint32_t here = ring(s), next = ring(s + 1);
            const uint32_t b1_here = b_addr[1] + here, b0_next = b_addr[0] + next, h_next = h_addr + next;
#pragma unroll
            for (int j = 0; j < 32; ++j) {
                const int kk = j >> 4, n = (j >> 1) & 7, m = j & 1;
                if (j == 16) {                                  // this step's second half, and the next step's words and h
                    wait_lds();
                    touch_b(1);
                    touch_h();
#pragma unroll
                    for (int mm = 0; mm < MP; ++mm)
#pragma unroll
                        for (int k = 0; k < K; ++k) sign_a(mm, k);
                }
                acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[p][m][kk], b[n][kk], acc[m][n], 0, 0, 0);
                if (j == 0) {
                    // the copies of step s + 1 were requested NBUF - 2 steps before it, and
                    // CP * (NBUF - 3) copies came after them; behind the barrier every wavefront has
                    // read what it needed from the buffer of step s - 1, which the next copies fill
                    wait_copies_and_sync<CP * (NBUF - 3)>();
                    stage_step(s + NBUF - 1);
                }
                if (j < 8) read_b(b1_here, j, 1);
                if (j >= 1 && j < 2 * K + 2) read_h(h_next, j - 1);
                if (j >= 8 && j < 8 + MP * K) fetch_a(cur, c_, q_, (j - 8) / K, (j - 8) % K);
                if (j >= 16 && j < 24) read_b(b0_next, j - 16, 0);
                if (j >= 16) expand_a(j - 16, a[pn]);
                __builtin_amdgcn_sched_barrier(0);
            }
            wait_lds();
            touch_b(0);
            // the words of column half c were last fetched for its fourth step, one step ahead
            if ((step & 3) == 2 && ct + 1 < ct_end) reload_half(ct + 1, step >> 2, cur);
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // no copy may land in LDS after the end

    // ---- epilogue: lane l of tile (m, n) holds token 32n + l % 32 and, in register 4a + e, row
    // 8a + 4 (l / 32) + e of the 32
    asm volatile("" : "+s"(out));
    const float inv_s = scl[6];
#pragma unroll
    for (int n = 0; n < NT; ++n) {
        const int t = tb * BLK_TOK + n * 32 + (lane & 31);
        if (t >= T) continue;
#pragma unroll
        for (int m = 0; m < MP; ++m) {
#pragma unroll
            for (int a4 = 0; a4 < 4; ++a4) {
                const int row0 = (rt_base + 2 * m) * TILE_ROWS + 8 * a4 + 4 * kg;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (row0 + e >= out) continue;
                    if (partial)
                        Acc[((size_t)slice * T + t) * tail_rows + (row0 + e - tail_row0)] = acc[m][n][4 * a4 + e];
                    else
                        store_out(Y, OUT_DT, (size_t)t * out + row0 + e, acc[m][n][4 * a4 + e] * inv_s);
                }
            }
        }
    }
}

// ------------------------------------------------------------------ host ---
struct Plan {
    bool small;          // 32-token tiles with the contraction split over workgroups
    int T_pad, CT, in_pad, RT, RB, TB, split;
    // 256-token tiles: the tiles of the last, partly filled round are shared by tail_split workgroups each
    int full_tiles, tail_split, tail_row0, tail_rows;
    size_t u_bytes, acc_bytes;
    size_t hblk_bytes;   // 256-token tiles (one contraction): the h blocks; u_bytes then holds X in fp16
};

static Plan make_plan(const rb_layer *L, int T)
{
    Plan p;
    p.small = T <= SMALL_TOKENS && L->K == 2;       // three paths: the one-contraction kernel at any token count
    const int blk_tok = p.small ? SMALL_TOKENS : LARGE_TOKENS;
    p.T_pad = round_up(T, blk_tok);
    p.CT = col_tiles(L->in);
    p.in_pad = p.CT * TILE_COLS;
    p.RT = row_tiles(L->out);
    p.RB = (p.RT + BLK_ROWS / TILE_ROWS - 1) / (BLK_ROWS / TILE_ROWS);
    p.TB = p.T_pad / blk_tok;
    // enough workgroups for every compute unit of an MI355X (256), never less than one column tile each
    p.split = p.small ? std::max(1, std::min(p.CT, (256 + p.RB * p.TB - 1) / (p.RB * p.TB))) : 1;
    p.hblk_bytes = p.small ? 0 : (size_t)p.CT * 8 * HBLOCK_BYTES;
    p.u_bytes = ((p.small ? 2 : 1) * (size_t)p.T_pad * p.in_pad * sizeof(_Float16) + 255) / 256 * 256;
    p.acc_bytes = p.split > 1 ? (size_t)p.split * T * L->out * sizeof(float) : 0;
    const int tiles = p.RB * p.TB;
    p.full_tiles = tiles;
    p.tail_split = 1;
    p.tail_row0 = 0;
    p.tail_rows = L->out;
    if (!p.small) {
        // A tile takes the same time wherever it runs, so a last round that fills half of the
        // compute units or less costs a whole round.  Its tiles (whole row blocks) are cut along
        // the contraction instead, into as many slices as fill the round.
        const int cus = mx::device_groups();
        const int G = cus > 0 ? cus : 256;               // no device (size queries on a host): an MI355X
        const int full = tiles / G * G / p.TB * p.TB;
        const int tail = tiles - full;
        const int cut = tail > 0 ? std::min(std::min(G / tail, 4), p.CT) : 1;
        if (cut > 1) {
            p.full_tiles = full;
            p.tail_split = cut;
            p.tail_row0 = full / p.TB * BLK_ROWS;
            p.tail_rows = L->out - p.tail_row0;
            p.acc_bytes = (size_t)cut * T * p.tail_rows * sizeof(float);
        }
    }
    return p;
}

size_t workspace_bytes(const rb_layer *L, int T)
{
    const Plan p = make_plan(L, T);
    return SCALES_BYTES + p.hblk_bytes + p.u_bytes + p.acc_bytes;
}

bool supported(const rb_layer *L, int T)
{
    return (L->K == 2 || L->K == 3) && T >= 1;
}

int launch(const rb_layer *L, const void *X, void *Y, int T, int act_dtype, int out_dtype, void *workspace,
           hipStream_t stream)
{
    const Plan p = make_plan(L, T);
    float *scl = static_cast<float *>(workspace);
    uint8_t *Hblk = static_cast<uint8_t *>(workspace) + SCALES_BYTES;
    _Float16 *U = reinterpret_cast<_Float16 *>(Hblk + p.hblk_bytes);
    float *Acc = p.acc_bytes > 0 ? reinterpret_cast<float *>(reinterpret_cast<uint8_t *>(U) + p.u_bytes) : nullptr;
    const __half *h = reinterpret_cast<const __half *>(L->h);
    const dim3 sgrid(p.in_pad / 256, p.T_pad);
    if (!p.small) {
        // one contraction on the effective weight built in registers
        const uint32_t *bits = static_cast<const uint32_t *>(L->bits);
        const __half *g = reinterpret_cast<const __half *>(L->g);
        static_assert(ABSMAX_GROUPS == 64 && ABSMAX_GROUPS * 8 * sizeof(float) <= LARGE_TOKENS * TILE_COLS * sizeof(_Float16), "partials fit in U");
        hipLaunchKernelGGL(absmax_kernel, dim3(ABSMAX_GROUPS), dim3(256), 0, stream, g, h, L->K, L->out, L->in, reinterpret_cast<float *>(U));
        hipLaunchKernelGGL(scales1_kernel, dim3(1), dim3(64), 0, stream, reinterpret_cast<const float *>(U), L->K, scl);
        hipLaunchKernelGGL(hblock_kernel, dim3(p.CT * 8), dim3(32 * RB_MAX_K), 0, stream, h, scl, L->K, L->in, Hblk);
        const dim3 xgrid((p.in_pad / 8 + 255) / 256, p.T_pad);
        if (act_dtype == RB_F16)
            hipLaunchKernelGGL(xperm_kernel<__half>, xgrid, dim3(256), 0, stream, static_cast<const __half *>(X), U, T, p.T_pad,
                               L->in, p.in_pad);
        else
            hipLaunchKernelGGL(xperm_kernel<bf16_t>, xgrid, dim3(256), 0, stream, static_cast<const bf16_t *>(X), U, T, p.T_pad,
                               L->in, p.in_pad);
        const int tail_tiles = p.RB * p.TB - p.full_tiles;
        const dim3 grid((unsigned)(p.full_tiles + tail_tiles * p.tail_split));
        constexpr int lds1 = ONE_NBUF * ONE_BUF_BYTES;
        auto run = [&](auto kernel) -> int {
            if (hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, lds1) !=
                hipSuccess)
                return RB_ERR_HIP;
            hipLaunchKernelGGL(kernel, grid, dim3(256), lds1, stream, bits, g, scl, Hblk, U, Y, Acc, L->out, p.RT, p.CT, T, p.T_pad,
                               p.full_tiles, p.tail_split, p.tail_row0, p.tail_rows);
            return RB_OK;
        };
        const int rc = L->K == 3 ? (out_dtype == RB_F16    ? run(gemm1_kernel<RB_F16, 3>)
                                    : out_dtype == RB_BF16 ? run(gemm1_kernel<RB_BF16, 3>)
                                                           : run(gemm1_kernel<RB_F32, 3>))
                                 : (out_dtype == RB_F16    ? run(gemm1_kernel<RB_F16, 2>)
                                    : out_dtype == RB_BF16 ? run(gemm1_kernel<RB_BF16, 2>)
                                                           : run(gemm1_kernel<RB_F32, 2>));
        if (rc != RB_OK) return rc;
        if (p.tail_split > 1) {
            const size_t n = (size_t)T * p.tail_rows;
            hipLaunchKernelGGL(finish_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, Acc, scl, Y, out_dtype, T,
                               L->out, p.tail_row0, p.tail_rows, p.tail_split, 6);
        }
        return hipGetLastError() == hipSuccess ? RB_OK : RB_ERR_HIP;
    }
    hipLaunchKernelGGL(hscale_kernel, dim3(1), dim3(256), 0, stream, h, L->in, scl);
    if (act_dtype == RB_F16)
        hipLaunchKernelGGL(scale_kernel<__half>, sgrid, dim3(256), 0, stream, static_cast<const __half *>(X), h, scl, U,
                           T, p.T_pad, L->in, p.in_pad);
    else
        hipLaunchKernelGGL(scale_kernel<bf16_t>, sgrid, dim3(256), 0, stream, static_cast<const bf16_t *>(X), h, scl, U,
                           T, p.T_pad, L->in, p.in_pad);
    const v4u *bits = static_cast<const v4u *>(L->bits);
    const __half *g = reinterpret_cast<const __half *>(L->g);
    const int tail_tiles = p.RB * p.TB - p.full_tiles;
    const dim3 grid((unsigned)(p.full_tiles + tail_tiles * p.tail_split), (unsigned)p.split);
    const size_t lds = p.small ? (size_t)(AHEAD_SMALL + 1) * SMALL_TOKENS * 64 : (size_t)(AHEAD_LARGE + 1) * LARGE_TOKENS * 64;
#define RB_GEMM(DT, WM, WN, MP, NT)                                                                              \
    hipLaunchKernelGGL((gemm_kernel<DT, WM, WN, MP, NT, (NT == 1 ? AHEAD_SMALL : AHEAD_LARGE)>), grid, dim3(256), lds, \
                       stream, bits, g, scl, U, Y, Acc, L->out, p.RT, p.CT, T, p.T_pad, p.full_tiles, p.tail_split, p.tail_row0, \
                       p.tail_rows)
    if (p.small && p.split > 1) {
        RB_GEMM(RB_F32, 4, 1, 2, 1);
        const size_t n = (size_t)T * L->out;
        hipLaunchKernelGGL(finish_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, Acc, scl, Y, out_dtype, T,
                           L->out, 0, L->out, p.split, 4);
    } else {
        if (out_dtype == RB_F16) RB_GEMM(RB_F16, 4, 1, 2, 1);
        else if (out_dtype == RB_BF16) RB_GEMM(RB_BF16, 4, 1, 2, 1);
        else RB_GEMM(RB_F32, 4, 1, 2, 1);
    }
#undef RB_GEMM
    return hipGetLastError() == hipSuccess ? RB_OK : RB_ERR_HIP;
}

}  // namespace gemm
}  // namespace rb
