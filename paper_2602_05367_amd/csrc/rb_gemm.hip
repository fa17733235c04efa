// Many-token path of the residual-binary layer: a matrix-core GEMM.
//
// Section 4.1 / Eq. (stacked binary weight): Y[t][i] = sum_k g_k[i] * sum_j B_k[i][j] * (h_k[j] X[t][j]).
// With T in the thousands this is a dense contraction and belongs on the MFMA units:
//   * a pre-pass forms U_k = h_k (.) X once, in fp16 (input scaling, Section 4.1);
//   * the GEMM contracts over the pair (path, input column) with a single accumulator: the left
//     operand element for row i is +-g_k[i] (an exact fp16 value: the stored scale with the sign
//     bit of the weight), the right operand is U_k.  Both paths land in the same fp32 sum, so
//     the path sum of Eq. (stacked binary weight) costs nothing;
//   * the left operand never exists in memory: each wavefront turns the packed sign words of its
//     rows into v_mfma_f32_16x16x32_f16 operand registers with two vector instructions per
//     register (shift so that two sign bits land on bits 15 and 31, then and-or with the packed
//     pair of |g|).  Inside a group of 32 columns the order of the contraction index is free as
//     long as both operands agree; the pre-pass stores U in the order this shift produces:
//     position 2n + hi holds the column whose sign is native bit n + 16 * hi of the word;
//   * the right operand goes through LDS (double buffered, one barrier per 32 columns), shared by
//     the four wavefronts of a 256-row x 256-token workgroup tile; a wavefront owns 128 x 128 of
//     it in 64 accumulator tiles.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include "rabit.h"
#include "rb_device.h"
#include "rb_internal.h"
#include "rb_layout.h"

namespace rb {
namespace gemm {

typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef unsigned v4u __attribute__((ext_vector_type(4)));

constexpr int BLK = 256;            // rows and tokens of a workgroup tile
constexpr int LDS_STRIDE = 40;      // halves per token row in LDS: 32 of data + 8 of padding (bank spread)

__host__ __device__ inline int round_up(int v, int a) { return (v + a - 1) / a * a; }

// position inside a group of 32 columns at which the pre-pass stores column `col` (0..31)
__host__ __device__ inline int contraction_position(int col)
{
    const int b = native_bit(col);  // bit of the native sign word
    return 2 * (b & 15) + (b >> 4);
}

// ------------------------------------------------------------- pre-pass ---
// U[k][t][j'] = fp16(h_k[j] * X[t][j]); rows t >= T and columns j >= in are zero.
template <typename ActT>
__global__ __launch_bounds__(256) void scale_kernel(const ActT *__restrict__ X, const __half *__restrict__ h,
                                                    _Float16 *__restrict__ U, int T, int T_pad, int in, int in_pad)
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
        U[((size_t)k * T_pad + t) * in_pad + jp] = (_Float16)(hv * x);
    }
}

// ----------------------------------------------------------------- GEMM ---
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

template <int OUT_DT>
__global__ __launch_bounds__(256, 1) void gemm_kernel(const v4u *__restrict__ bits, const __half *__restrict__ g,
                                                      const _Float16 *__restrict__ U, void *__restrict__ Y,
                                                      int out, int RT, int CT, int T, int T_pad)
{
    __shared__ __attribute__((aligned(16))) _Float16 Bs[2][BLK * LDS_STRIDE];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave & 1, wn = wave >> 1;
    const int r = lane & 15, kg = lane >> 4;
    const int in_pad = CT * TILE_COLS;
    // workgroups that share a token block sit on the same XCD (ids are dealt round-robin over
    // eight of them), so the slice of U they all walk stays in that XCD's L2
    const int TB = T_pad / BLK;
    const int tb = blockIdx.x % TB, rb = blockIdx.x / TB;

    // ---- per-row constants: |g| as a packed pair, and whether the sign bits must be flipped
    uint32_t G2[8][2], flip[8][2];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int row = (rb * 16 + wm * 8 + i) * TILE_ROWS + r;
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            const uint32_t gb = row < out ? (uint32_t)__half_as_ushort(g[(size_t)k * out + row]) : 0u;
            const uint32_t mag = gb & 0x7fffu;
            G2[i][k] = mag | (mag << 16);
            flip[i][k] = (gb & 0x8000u) ? 0xffffffffu : 0u;
        }
    }
    // lane (r, kg) takes columns 8kg..8kg+7 of the step: register i gets native bits n and n + 16,
    // n = 4kg + i, on bits 15 and 31
    uint32_t sh[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) sh[i] = (uint32_t)(15 - 4 * kg - i);

    // sign words of this wavefront's eight row tiles for one column tile: lane (r, q) holds, for row
    // r, the four words [column half c][path k] of columns 128c + 32q .. +31
    auto load_words = [&](int ct, v4u (&w)[8]) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int rt = rb * 16 + wm * 8 + i;
            v4u v = {0u, 0u, 0u, 0u};
            if (rt < RT) v = bits[((size_t)rt * CT + ct) * 64 + lane];
            v[0] ^= flip[i][0]; v[1] ^= flip[i][1]; v[2] ^= flip[i][0]; v[3] ^= flip[i][1];
            w[i] = v;
        }
    };

    // right-operand staging: thread -> (token tid / 4 + 64 j, 16-byte chunk tid % 4), j = 0..3
    const int st_tok = tid >> 2, st_chunk = tid & 3;
    const _Float16 *Ubase = U + ((size_t)tb * BLK + st_tok) * in_pad + st_chunk * 8;
    auto stage_load = [&](int k, int col0, v4u (&regs)[4]) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
            regs[j] = *reinterpret_cast<const v4u *>(Ubase + ((size_t)k * T_pad + 64 * j) * in_pad + col0);
    };
    auto stage_store = [&](int buf, const v4u (&regs)[4]) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
            *reinterpret_cast<v4u *>(&Bs[buf][(st_tok + 64 * j) * LDS_STRIDE + st_chunk * 8]) = regs[j];
    };

    v4f acc[8][8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int n = 0; n < 8; ++n) acc[i][n] = (v4f){0.f, 0.f, 0.f, 0.f};

    v4u cur[8], nxt[8];
    load_words(0, cur);
    v4u staged[4];
    stage_load(0, 0, staged);

    int buf = 0;
    for (int ct = 0; ct < CT; ++ct) {
        if (ct + 1 < CT) load_words(ct + 1, nxt);
#pragma unroll
        for (int step = 0; step < 16; ++step) {
            const int k = step >> 3, c = (step >> 2) & 1, q = step & 3;     // path, column half, 32-column group
            stage_store(buf, staged);
            {
                // request the right operand of the next step while this one is computed
                const int ns = step + 1;
                const int nct = ns < 16 ? ct : ct + 1;
                const int nk = (ns & 15) >> 3, ncq = ns & 7;
                if (nct < CT) stage_load(nk, nct * TILE_COLS + ncq * 32, staged);
            }
            lds_barrier();
            // left operand: every lane fetches the word of its row from lane (r, q), then expands
            // its quarter of the 32 columns
            v8h a[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const uint32_t w = (uint32_t)__shfl((int)cur[i][c * 2 + k], r + 16 * q);
                union { uint32_t u[4]; v8h h; } f;
#pragma unroll
                for (int e = 0; e < 4; ++e) f.u[e] = ((w << sh[e]) & 0x80008000u) | G2[i][k];
                a[i] = f.h;
            }
#pragma unroll
            for (int n = 0; n < 8; ++n) {
                const v8h b = *reinterpret_cast<const v8h *>(&Bs[buf][(wn * 128 + n * 16 + r) * LDS_STRIDE + kg * 8]);
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    acc[i][n] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[i], b, acc[i][n], 0, 0, 0);
            }
            buf ^= 1;
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) cur[i] = nxt[i];
    }

    // ---- epilogue: lane (r, kg) of tile (i, n) holds token 16n + r, rows 4kg .. 4kg + 3
#pragma unroll
    for (int n = 0; n < 8; ++n) {
        const int t = tb * BLK + wn * 128 + n * 16 + r;
        if (t >= T) continue;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int row0 = (rb * 16 + wm * 8 + i) * TILE_ROWS + 4 * kg;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (row0 + e < out) store_out(Y, OUT_DT, (size_t)t * out + row0 + e, acc[i][n][e]);
        }
    }
}

size_t workspace_bytes(const rb_layer *L, int T)
{
    const size_t T_pad = (size_t)round_up(T, BLK), in_pad = (size_t)col_tiles(L->in) * TILE_COLS;
    return 2 * T_pad * in_pad * sizeof(_Float16);
}

bool supported(const rb_layer *L, int T)
{
    return L->K == 2 && T >= 1;
}

int launch(const rb_layer *L, const void *X, void *Y, int T, int act_dtype, int out_dtype, void *workspace,
           hipStream_t stream)
{
    const int T_pad = round_up(T, BLK), CT = col_tiles(L->in), in_pad = CT * TILE_COLS, RT = row_tiles(L->out);
    _Float16 *U = static_cast<_Float16 *>(workspace);
    const __half *h = reinterpret_cast<const __half *>(L->h);
    const dim3 sgrid(in_pad / 256, T_pad);
    if (act_dtype == RB_F16)
        hipLaunchKernelGGL(scale_kernel<__half>, sgrid, dim3(256), 0, stream, static_cast<const __half *>(X), h, U,
                           T, T_pad, L->in, in_pad);
    else
        hipLaunchKernelGGL(scale_kernel<bf16_t>, sgrid, dim3(256), 0, stream, static_cast<const bf16_t *>(X), h, U,
                           T, T_pad, L->in, in_pad);
    const int RB = (RT + 15) / 16, TB = T_pad / BLK;
    const dim3 grid((unsigned)(RB * TB));
    const v4u *bits = static_cast<const v4u *>(L->bits);
    const __half *g = reinterpret_cast<const __half *>(L->g);
#define RB_GEMM(DT) \
    hipLaunchKernelGGL(gemm_kernel<DT>, grid, dim3(256), 0, stream, bits, g, U, Y, L->out, RT, CT, T, T_pad)
    if (out_dtype == RB_F16) RB_GEMM(RB_F16);
    else if (out_dtype == RB_BF16) RB_GEMM(RB_BF16);
    else RB_GEMM(RB_F32);
#undef RB_GEMM
    return hipGetLastError() == hipSuccess ? RB_OK : RB_ERR_HIP;
}

}  // namespace gemm
}  // namespace rb
