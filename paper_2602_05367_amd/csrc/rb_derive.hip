// Initialisation of the paths from a full-precision weight (Section 4.3, Alg. 1): Iterative
// Residual SVID on the preconditioned weight W' = rows (.) W (.) cols (Eq. init-calib).
//
//   What_i = 0;  for t = 1..T_max, for i = 1..K:
//       R_i = W' - sum_{j != i} What_j        (Eq. init-iter; paths j < i of this sweep, j > i of the last)
//       B_i = sign(R_i);  (sigma, a, b) = leading singular triplet of |R_i|
//       g_i' = sqrt(sigma) a,  h_i' = sqrt(sigma) b;  What_i = g_i' (.) B_i (.) h_i'
//   g_i = g_i' / rows,  h_i = h_i' / cols
//
// Everything is fp64 (the sign of a residual decides a stored bit).  No residual and no What_i is
// ever materialised: a path is its packed signs and two vectors, and every pass recomputes R_i
// from W (4 bytes per weight) and the other paths (a bit and two cached scale values each), so a
// pass is bound by the HBM read of W.  The singular triplet comes from a power iteration from the
// all-ones vector (the matrix is non-negative): two passes per iteration, a = |R| b by rows (one
// wavefront per row) and b = |R|^T a by columns (slices of rows, partial sums added in slice
// order); in both a lane takes four consecutive columns, one 16-byte load of W.  Every sum has a fixed order.  The iteration's stopping rule is
// evaluated on the device; the host reads one flag every few iterations, so the call synchronises.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "rabit.h"
#include "rb_device.h"
#include "rb_internal.h"

namespace rb {
namespace derive {

constexpr int ROW_SLICE = 64;          // rows one workgroup of the column pass walks
constexpr int CHECK_EVERY = 4;         // power iterations between two looks at the flag
constexpr int MAX_ITER = 200;
constexpr double TOL_SIGMA = 1e-13, TOL_B = 1e-10;

struct Problem {
    const float *W;
    const double *rows, *cols;         // preconditioning factors (nullptr: 1)
    const uint32_t *packed;            // [K][out][in/32]
    const double *g, *h;               // [K][out], [K][in]: g', h' of the preconditioned domain
    int K, out, in;
};

// R_i[r][c .. c + 3] for path `skip` (skip < 0: the error of the whole approximation, no path left
// out); c % 4 == 0.  One 16-byte load of W, four bits of one sign word per path.
__device__ __forceinline__ void residual4(const Problem &p, int r, int c, int skip, const double *g_r, double rows_r,
                                          double v[4])
{
    const float4 w = *reinterpret_cast<const float4 *>(p.W + (size_t)r * p.in + c);
    v[0] = (double)w.x; v[1] = (double)w.y; v[2] = (double)w.z; v[3] = (double)w.w;
    if (p.rows)
        for (int e = 0; e < 4; ++e) v[e] = rows_r * v[e];
    if (p.cols) {
        const double2 c01 = *reinterpret_cast<const double2 *>(p.cols + c), c23 = *reinterpret_cast<const double2 *>(p.cols + c + 2);
        v[0] = v[0] * c01.x; v[1] = v[1] * c01.y; v[2] = v[2] * c23.x; v[3] = v[3] * c23.y;
    }
    const int W32 = p.in / 32;
    for (int j = 0; j < p.K; ++j) {
        if (j == skip) continue;
        const uint32_t bits4 = p.packed[((size_t)j * p.out + r) * W32 + (c >> 5)] >> (c & 31);
        const double2 h01 = *reinterpret_cast<const double2 *>(p.h + (size_t)j * p.in + c);
        const double2 h23 = *reinterpret_cast<const double2 *>(p.h + (size_t)j * p.in + c + 2);
        const double hv[4] = {h01.x, h01.y, h23.x, h23.y};
        for (int e = 0; e < 4; ++e) {
            const double gs = (bits4 >> e) & 1u ? -g_r[j] : g_r[j];
            v[e] -= gs * hv[e];
        }
    }
}

struct Scalars {
    double sigma;       // the iteration's current estimate (norm of |R|^T a)
    double na;          // norm of |R| b
    double db;          // norm of the last change of b
    int done;           // the stopping rule held (or the matrix is zero)
    int zero;           // |R| b = 0
    int iters;
    int pad_;
};

// one workgroup: sum of squares of v[0..n) in a fixed order
__device__ double block_sumsq(const double *v, int n, double *red)
{
    double s = 0.0;
    for (int i = threadIdx.x; i < n; i += blockDim.x) s += v[i] * v[i];
    red[threadIdx.x] = s;
    __syncthreads();
    for (int w = blockDim.x / 2; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
        __syncthreads();
    }
    const double total = red[0];
    __syncthreads();
    return total;
}

__global__ __launch_bounds__(256) void start_kernel(double *b, int in, Scalars *sc)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < in) b[i] = 1.0 / sqrt((double)in);
    if (i == 0) {
        sc->sigma = 0.0; sc->na = 0.0; sc->db = 0.0; sc->done = 0; sc->zero = 0; sc->iters = 0; sc->pad_ = 0;
    }
}

// a_raw[r] = sum_c |R[r][c]| b[c]; one wavefront per row, a lane takes four consecutive columns at
// a time (256 columns per step of the wavefront)
__global__ __launch_bounds__(256) void rows_kernel(Problem p, int skip, const double *b, double *a_raw, const Scalars *sc,
                                                   bool final_pass)
{
    if (!final_pass && sc->done) return;
    const int lane = threadIdx.x & 63;
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= p.out) return;
    double g_r[RB_MAX_K];
    for (int j = 0; j < p.K; ++j) g_r[j] = p.g[(size_t)j * p.out + r];
    const double rows_r = p.rows ? p.rows[r] : 1.0;
    double s = 0.0;
#pragma unroll 2
    for (int c = 4 * lane; c < p.in; c += 256) {
        double v[4];
        residual4(p, r, c, skip, g_r, rows_r, v);
        const double2 b01 = *reinterpret_cast<const double2 *>(b + c), b23 = *reinterpret_cast<const double2 *>(b + c + 2);
        s += fabs(v[0]) * b01.x;
        s += fabs(v[1]) * b01.y;
        s += fabs(v[2]) * b23.x;
        s += fabs(v[3]) * b23.y;
    }
    for (int m = 32; m > 0; m >>= 1) s += __shfl_xor(s, m);
    if (lane == 0) a_raw[r] = s;
}

// a = a_raw / ||a_raw||  (one workgroup)
__global__ __launch_bounds__(1024) void unit_a_kernel(const double *a_raw, double *a, int out, Scalars *sc, bool final_pass)
{
    if (!final_pass && sc->done) return;
    __shared__ double red[1024];
    const double na = sqrt(block_sumsq(a_raw, out, red));
    for (int i = threadIdx.x; i < out; i += 1024) a[i] = na > 0.0 ? a_raw[i] / na : 0.0;
    if (threadIdx.x == 0) {
        sc->na = na;
        if (na == 0.0) { sc->zero = 1; sc->done = 1; }
    }
}

// partial[slice][c] = sum over the slice's rows of |R[r][c]| a[r]; a thread per four consecutive
// columns, the rows of the slice in order
__global__ __launch_bounds__(64) void cols_kernel(Problem p, int skip, const double *a, double *partial, const Scalars *sc)
{
    if (sc->done) return;
    const int c = (blockIdx.x * 64 + threadIdx.x) * 4;
    const int r0 = blockIdx.y * ROW_SLICE, r1 = min(p.out, r0 + ROW_SLICE);
    if (c >= p.in) return;
    double s[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll 8
    for (int r = r0; r < r1; ++r) {
        double g_r[RB_MAX_K];
        for (int j = 0; j < p.K; ++j) g_r[j] = p.g[(size_t)j * p.out + r];
        double v[4];
        residual4(p, r, c, skip, g_r, p.rows ? p.rows[r] : 1.0, v);
        const double a_r = a[r];
        for (int e = 0; e < 4; ++e) s[e] += fabs(v[e]) * a_r;
    }
    double *dst = partial + (size_t)blockIdx.y * p.in + c;
    *reinterpret_cast<double2 *>(dst) = make_double2(s[0], s[1]);
    *reinterpret_cast<double2 *>(dst + 2) = make_double2(s[2], s[3]);
}

// sum[c] = the slices of partial[.][c] in order
__global__ __launch_bounds__(256) void slices_kernel(const double *partial, int n_slices, int in, double *sum, const Scalars *sc)
{
    if (sc->done) return;
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= in) return;
    double s = 0.0;
#pragma unroll 8
    for (int k = 0; k < n_slices; ++k) s += partial[(size_t)k * in + c];
    sum[c] = s;
}

// b_new = scratch / its norm, the change of b, the stopping rule  (one workgroup; scratch is used up)
__global__ __launch_bounds__(1024) void unit_b_kernel(double *b, double *scratch, int in, Scalars *sc)
{
    if (sc->done) return;
    __shared__ double red[1024];
    const double s_new = sqrt(block_sumsq(scratch, in, red));
    for (int c = threadIdx.x; c < in; c += 1024) {
        const double bn = scratch[c] / s_new;
        scratch[c] = bn - b[c];
        b[c] = bn;
    }
    __syncthreads();
    const double db = sqrt(block_sumsq(scratch, in, red));
    if (threadIdx.x == 0) {
        const bool done = fabs(s_new - sc->sigma) <= TOL_SIGMA * s_new && db <= TOL_B;
        sc->sigma = s_new;
        sc->db = db;
        sc->iters += 1;
        if (done || sc->iters >= MAX_ITER) sc->done = 1;
    }
}

// after the final a = |R| b: g' = sqrt(sigma) a / sigma, h' = sqrt(sigma) b with sigma = ||a_raw||
__global__ __launch_bounds__(1024) void scales_kernel(const double *a_raw, const double *b, double *g_i, double *h_i, int out, int in)
{
    __shared__ double red[1024];
    const double sigma = sqrt(block_sumsq(a_raw, out, red));
    const double root = sqrt(sigma);
    for (int i = threadIdx.x; i < out; i += 1024) g_i[i] = sigma > 0.0 ? root * (a_raw[i] / sigma) : 0.0;
    for (int i = threadIdx.x; i < in; i += 1024) h_i[i] = root * b[i];
}

// B_i = sign(R_i) (sign(0) = +1), packed 32 columns per word, bit b = column 32 w + b, 1 means -1.
// Written to a buffer of its own: the other kernels of this step still read path i's old signs
// nowhere (it is the path left out), but a wavefront must not read words another has replaced.
// Eight lanes hold the 32 columns of a word, four each: every lane shifts its four bits into place
// and an OR over the eight gives the word.
__global__ __launch_bounds__(256) void sign_kernel(Problem p, int skip, uint32_t *words)
{
    const int lane = threadIdx.x & 63;
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= p.out) return;
    double g_r[RB_MAX_K];
    for (int j = 0; j < p.K; ++j) g_r[j] = p.g[(size_t)j * p.out + r];
    const double rows_r = p.rows ? p.rows[r] : 1.0;
    const int W32 = p.in / 32;
    for (int c0 = 0; c0 < p.in; c0 += 256) {
        const int c = c0 + 4 * lane;
        uint32_t four = 0;
        if (c < p.in) {                                        // in % 32 == 0: all four columns or none
            double v[4];
            residual4(p, r, c, skip, g_r, rows_r, v);
            for (int e = 0; e < 4; ++e) four |= !(v[e] >= 0.0) ? 1u << e : 0u;
        }
        const uint32_t word = or_over_8(four << (4 * (lane & 7)));
        const int w = (c0 >> 5) + (lane >> 3);
        if ((lane & 7) == 0 && w < W32) words[(size_t)r * W32 + w] = word;
    }
}

// squared Frobenius norm of W' - sum_j What_j by rows, then one workgroup adds the rows up
__global__ __launch_bounds__(256) void err_rows_kernel(Problem p, double *row_sq)
{
    const int lane = threadIdx.x & 63;
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= p.out) return;
    double g_r[RB_MAX_K];
    for (int j = 0; j < p.K; ++j) g_r[j] = p.g[(size_t)j * p.out + r];
    const double rows_r = p.rows ? p.rows[r] : 1.0;
    double s = 0.0;
#pragma unroll 2
    for (int c = 4 * lane; c < p.in; c += 256) {
        double v[4];
        residual4(p, r, c, -1, g_r, rows_r, v);
        for (int e = 0; e < 4; ++e) s += v[e] * v[e];
    }
    for (int m = 32; m > 0; m >>= 1) s += __shfl_xor(s, m);
    if (lane == 0) row_sq[r] = s;
}
__global__ __launch_bounds__(1024) void err_sum_kernel(const double *row_sq, int out, double *err)
{
    __shared__ double red[1024];
    double s = 0.0;
    for (int i = threadIdx.x; i < out; i += 1024) s += row_sq[i];
    red[threadIdx.x] = s;
    __syncthreads();
    for (int w = 512; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) *err = sqrt(red[0]);
}

__global__ __launch_bounds__(256) void clear_kernel(double *v, size_t n, uint32_t *w, size_t nw)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) v[i] = 0.0;
    if (i < nw) w[i] = 0u;
}

// step 3: back to the original domain
__global__ __launch_bounds__(256) void unscale_kernel(double *g, double *h, const double *rows, const double *cols, int K, int out,
                                                      int in)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    for (int k = 0; k < K; ++k) {
        if (rows && i < out) g[(size_t)k * out + i] /= rows[i];
        if (cols && i < in) h[(size_t)k * in + i] /= cols[i];
    }
}

struct Layout {
    size_t scalars, a_raw, a, b, scratch, partial, words, row_sq, total;
};
static Layout make_layout(int out, int in)
{
    auto up = [](size_t v) { return (v + 255) / 256 * 256; };
    const size_t slices = (size_t)(out + ROW_SLICE - 1) / ROW_SLICE;
    Layout L;
    size_t o = 0;
    L.scalars = o; o += up(sizeof(Scalars));
    L.a_raw = o; o += up(sizeof(double) * out);
    L.a = o; o += up(sizeof(double) * out);
    L.b = o; o += up(sizeof(double) * in);
    L.scratch = o; o += up(sizeof(double) * in);
    L.partial = o; o += up(sizeof(double) * slices * in);
    L.words = o; o += up(sizeof(uint32_t) * (size_t)out * (in / 32));
    L.row_sq = o; o += up(sizeof(double) * out);
    L.total = o;
    return L;
}

}  // namespace derive
}  // namespace rb

extern "C" size_t rb_derive_workspace_bytes(int out, int in)
{
    if (out < 1 || in < 32 || in % 32 != 0) return 0;
    return rb::derive::make_layout(out, in).total;
}

extern "C" int rb_derive_iterative(const float *W, const double *row_factors, const double *col_factors, int K, int T_max,
                                   int out, int in, uint32_t *packed, double *g, double *h, double *err, void *workspace,
                                   size_t workspace_bytes, void *stream_)
{
    using namespace rb::derive;
    if (!W || !packed || !g || !h) return RB_ERR_NULL;
    if (K < 1 || K > RB_MAX_K || T_max < 1 || out < 1 || in < 32 || in % 32 != 0) return RB_ERR_SHAPE;
    if ((uintptr_t)packed & 3) return RB_ERR_ALIGN;
    if (((uintptr_t)g | (uintptr_t)row_factors | (uintptr_t)err) & 7) return RB_ERR_ALIGN;
    if (((uintptr_t)W | (uintptr_t)h | (uintptr_t)col_factors) & 15) return RB_ERR_ALIGN;      // read 16 bytes at a time
    const Layout lay = make_layout(out, in);
    if (!workspace || workspace_bytes < lay.total) return RB_ERR_WORKSPACE;
    if ((uintptr_t)workspace & 15) return RB_ERR_ALIGN;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    uint8_t *ws = static_cast<uint8_t *>(workspace);
    Scalars *sc = reinterpret_cast<Scalars *>(ws + lay.scalars);
    double *a_raw = reinterpret_cast<double *>(ws + lay.a_raw), *a = reinterpret_cast<double *>(ws + lay.a);
    double *b = reinterpret_cast<double *>(ws + lay.b), *scratch = reinterpret_cast<double *>(ws + lay.scratch);
    double *partial = reinterpret_cast<double *>(ws + lay.partial), *row_sq = reinterpret_cast<double *>(ws + lay.row_sq);
    uint32_t *words = reinterpret_cast<uint32_t *>(ws + lay.words);
    const int W32 = in / 32;
    const int n_slices = (out + ROW_SLICE - 1) / ROW_SLICE;
    const dim3 by_rows((out + 3) / 4), by_cols((in + 255) / 256, n_slices);      // the column pass: 64 threads of 4 columns

    // What_i^(0) = 0: zero scales (and all-plus signs, which the zero scales make irrelevant)
    const size_t nv = (size_t)K * std::max(out, in), nw = (size_t)K * out * W32;
    hipLaunchKernelGGL(clear_kernel, dim3((unsigned)((std::max(nv, nw) + 255) / 256)), dim3(256), 0, stream, g,
                       (size_t)K * out, packed, nw);
    hipLaunchKernelGGL(clear_kernel, dim3((unsigned)(((size_t)K * in + 255) / 256)), dim3(256), 0, stream, h, (size_t)K * in,
                       static_cast<uint32_t *>(nullptr), (size_t)0);
    Problem p{W, row_factors, col_factors, packed, g, h, K, out, in};

    for (int t = 0; t < T_max; ++t) {
        for (int i = 0; i < K; ++i) {
            hipLaunchKernelGGL(start_kernel, dim3((in + 255) / 256), dim3(256), 0, stream, b, in, sc);
            for (int it = 0; it < MAX_ITER; it += CHECK_EVERY) {
                for (int n = 0; n < CHECK_EVERY; ++n) {
                    hipLaunchKernelGGL(rows_kernel, by_rows, dim3(256), 0, stream, p, i, b, a_raw, sc, false);
                    hipLaunchKernelGGL(unit_a_kernel, dim3(1), dim3(1024), 0, stream, a_raw, a, out, sc, false);
                    hipLaunchKernelGGL(cols_kernel, by_cols, dim3(64), 0, stream, p, i, a, partial, sc);
                    hipLaunchKernelGGL(slices_kernel, dim3((in + 255) / 256), dim3(256), 0, stream, partial, n_slices, in, scratch, sc);
                    hipLaunchKernelGGL(unit_b_kernel, dim3(1), dim3(1024), 0, stream, b, scratch, in, sc);
                }
                Scalars host;
                if (hipMemcpyAsync(&host, sc, sizeof(host), hipMemcpyDeviceToHost, stream) != hipSuccess ||
                    hipStreamSynchronize(stream) != hipSuccess)
                    return RB_ERR_HIP;
                if (host.done) break;
            }
            // sigma and a for the converged b, the signs of R_i, then the path's new scales
            hipLaunchKernelGGL(rows_kernel, by_rows, dim3(256), 0, stream, p, i, b, a_raw, sc, true);
            hipLaunchKernelGGL(sign_kernel, by_rows, dim3(256), 0, stream, p, i, words);
            hipLaunchKernelGGL(scales_kernel, dim3(1), dim3(1024), 0, stream, a_raw, b, g + (size_t)i * out, h + (size_t)i * in, out,
                               in);
            if (hipMemcpyAsync(packed + (size_t)i * out * W32, words, sizeof(uint32_t) * (size_t)out * W32,
                               hipMemcpyDeviceToDevice, stream) != hipSuccess)
                return RB_ERR_HIP;
            if (err) {
                hipLaunchKernelGGL(err_rows_kernel, by_rows, dim3(256), 0, stream, p, row_sq);
                hipLaunchKernelGGL(err_sum_kernel, dim3(1), dim3(1024), 0, stream, row_sq, out, err + (size_t)t * K + i);
            }
        }
    }
    if (row_factors || col_factors)
        hipLaunchKernelGGL(unscale_kernel, dim3((std::max(out, in) + 255) / 256), dim3(256), 0, stream, g, h, row_factors,
                           col_factors, K, out, in);
    if (hipGetLastError() != hipSuccess) return RB_ERR_HIP;
    return hipStreamSynchronize(stream) == hipSuccess ? RB_OK : RB_ERR_HIP;
}
