// Matrix-core path: set-up kernels, the persistent stack kernel, and its host
// planner.  See rb_mx.h for the arithmetic and the operand layout.
//
// Work split of the persistent kernel (one workgroup per compute unit):
//   * every op's row tiles are cut into contiguous shares, one per workgroup;
//     a share is a contiguous run of 1 KB sign tiles in the native layout and
//     is cut again into eight runs, one per compute wavefront;
//   * a compute wavefront keeps RING_D sign tiles in flight from HBM into its
//     LDS ring (the weights of later ops do not depend on activations, so the
//     stream never stops at a stage boundary), reads the expanded input of the
//     current stage NB tiles ahead, and issues four MFMAs per tile;
//   * partial sums of the wavefronts that share a row tile meet in LDS;
//   * four more wavefronts finish rows: y = sum_k g_k * acc_k, fp16 rounding,
//     the store, the four-term expansion of h (.) y for the ops that read y
//     next, and the cross-CU hand-over (agent-scope stores, one flag per
//     workgroup, agent-scope polling).  Keeping this traffic on wavefronts of
//     their own means no wait on it ever drains a weight prefetch.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include <cmath>
#include <cstring>
#include <vector>

#include "rabit.h"
#include "rb_internal.h"
#include "rb_layout.h"
#include "rb_mx.h"

namespace rb {
namespace mx {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));

#define RB_LDS(p) ((__attribute__((address_space(3))) void *)(p))

// ---------------------------------------------------------------- helpers ---
__device__ __forceinline__ uint32_t lds_addr(const void *p)
{
    return (uint32_t)(size_t)RB_LDS(p);
}

// four bf8 terms of u: u ~= t0 + t1/8 + t2/64 + t3/512 (each term rounds the rest)
__device__ __forceinline__ uint32_t expand4(float u)
{
    uint32_t out = 0;
    float r = u;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int pk = __builtin_amdgcn_cvt_pk_bf8_f32(r, 0.f, 0, false);
        out |= (uint32_t)(pk & 0xff) << (8 * t);
        r = (r - __builtin_amdgcn_cvt_f32_bf8(pk, 0)) * 8.f;
    }
    return out;
}

// byte address of (token, path, term, input column j) in an op's expanded input
__device__ __forceinline__ size_t up_offset(int CB, int tok, int p, int t, int j)
{
    const int cb = j >> 7;
    return ((size_t)((tok >> 1) * CB + cb) * 16 + (8 * (tok & 1) + 4 * p + t)) * 128 + operand_byte(j & 127);
}

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *base, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
}

// ------------------------------------------------------------ prep kernel ---
// One workgroup per op: power-of-two scale of each path's input scales, and the
// zero fill of the expanded-input array (padding columns and unused operand
// columns must read as zero).  Workgroup 0 also resets the hand-over flags.
__global__ __launch_bounds__(256) void prep_kernel(Header *hdr, Op *ops, uint32_t *flags, uint32_t *error,
                                                   uint32_t *zero_page, int reset_flags)
{
    Op &op = ops[blockIdx.x];
    __shared__ float red[256];
    for (int p = 0; p < 2; ++p) {
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
            const float mx_ = red[0];
            float sc = 1.f;
            if (mx_ > 0.f && mx_ < INFINITY) {
                int e;
                frexpf(mx_, &e);                 // mx_ = f * 2^e, f in [0.5, 1)
                sc = ldexpf(1.f, -e - 1);        // mx_ * sc in [0.25, 0.5)
            }
            op.sc[p] = sc;
            op.inv_sc[p] = 1.f / sc;
        }
        __syncthreads();
    }
    const size_t n16 = up_bytes(op.in, hdr->T) / 16;
    uint4 *up = reinterpret_cast<uint4 *>(op.up);
    for (size_t i = threadIdx.x; i < n16; i += 256) up[i] = make_uint4(0, 0, 0, 0);
    if (blockIdx.x == 0) {
        if (reset_flags)
            for (int i = threadIdx.x; i < hdr->n_groups; i += 256) flags[i] = hdr->epoch0 - 1u;
        if (threadIdx.x < 32) zero_page[threadIdx.x] = 0;
        if (threadIdx.x == 0) *error = 0;
    }
}

// --------------------------------------------------------- expand kernel ---
// Input scaling u_k = h_k (.) x (Section 4.1) for ops whose input comes from
// outside the fused ops, written as four bf8 terms in operand order.
__global__ __launch_bounds__(256) void expand_kernel(const Header *hdr, const Op *ops, const int *which)
{
    const Op &op = ops[which[blockIdx.z]];
    const int tok = blockIdx.y;
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= op.in) return;
    const int CB = col_tiles(op.in) * 2;
    const float x = __half2float(reinterpret_cast<const __half *>(op.x)[(size_t)tok * op.in + j]);
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const float h = __half2float(reinterpret_cast<const __half *>(op.h)[(size_t)p * op.in + j]);
        const uint32_t terms = expand4(h * x * op.sc[p]);
#pragma unroll
        for (int t = 0; t < 4; ++t) op.up[up_offset(CB, tok, p, t, j)] = (uint8_t)(terms >> (8 * t));
    }
}

// ---------------------------------------------------------- stack kernel ---
struct Span { int u0, u1, rt0, nrt; };

// share of workgroup `grp` (of G) and compute wavefront `wave` in an op
__device__ __forceinline__ Span op_span(int RT, int CT, int grp, int G, int wave)
{
    // all inputs are wavefront-uniform; RT <= MAXSLOT * G keeps the products inside 32 bits
    Span s;
    s.rt0 = (int)((uint32_t)grp * (uint32_t)RT / (uint32_t)G);
    s.nrt = (int)((uint32_t)(grp + 1) * (uint32_t)RT / (uint32_t)G) - s.rt0;
    const uint32_t U = (uint32_t)(s.nrt * CT);
    s.u0 = (int)((uint32_t)wave * U / CWAVES);
    s.u1 = (int)((uint32_t)(wave + 1) * U / CWAVES);
    s.rt0 = __builtin_amdgcn_readfirstlane(s.rt0);
    s.nrt = __builtin_amdgcn_readfirstlane(s.nrt);
    s.u0 = __builtin_amdgcn_readfirstlane(s.u0);
    s.u1 = __builtin_amdgcn_readfirstlane(s.u1);
    return s;
}

// workgroup barrier that orders LDS only: the weight prefetch of a compute wavefront stays in
// flight across it (a full fence would wait for every outstanding global load)
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

__device__ __forceinline__ const uint8_t *uniform_ptr(const void *p)
{
    const uint64_t v = (uint64_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return reinterpret_cast<const uint8_t *>(((uint64_t)hi << 32) | lo);
}

__device__ __forceinline__ v4f mfma_signs(uint32_t w, v8i b, v4f acc, uint32_t c22, int scale_b)
{
    v8i a;
    a[0] = (int)(((w << 3) & 0x88888888u) | c22);
    a[1] = (int)(((w << 2) & 0x88888888u) | c22);
    a[2] = (int)(((w << 1) & 0x88888888u) | c22);
    a[3] = (int)((w & 0x88888888u) | c22);
    a[4] = 0; a[5] = 0; a[6] = 0; a[7] = 0;
    // A: fp4 (cbsz = 4), B: bf8 (blgp = 1); scale bytes are E8M0 exponents
    return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, acc, 4, 1, 0, 0x7f7f7f7f, 0, scale_b);
}

struct BTile { v4i r[4]; };   // two 128-column blocks x 32 bytes per lane

__global__ __launch_bounds__(THREADS, 1) void stack_kernel(const Header *__restrict__ hdr_p,
                                                           const Op *__restrict__ ops,
                                                           const Stage *__restrict__ stages,
                                                           uint32_t *__restrict__ flags,
                                                           uint32_t *__restrict__ error,
                                                           const uint32_t *__restrict__ zero_page)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    float *part = reinterpret_cast<float *>(lds + LDS_RING_BYTES);
    uint32_t *misc = reinterpret_cast<uint32_t *>(lds + LDS_RING_BYTES + LDS_PART_BYTES);

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int grp = blockIdx.x, G = gridDim.x;
    const int n_ops = hdr_p->n_ops, n_stages = hdr_p->n_stages, T = hdr_p->T;
    const uint32_t epoch0 = hdr_p->epoch0;

    for (int i = threadIdx.x; i < LDS_PART_BYTES / 4; i += THREADS) part[i] = 0.f;
    if (threadIdx.x == 0) misc[0] = 0;
    __syncthreads();

    if (wave < CWAVES) {
        // ======================= compute wavefront ==========================
        uint8_t *ring = lds + wave * (RING_D * 1024);
        const int col = lane & 15, qd = lane >> 4;
        const int ncols = T > 1 ? 16 : 8;
        const int scale_b = (127 - 3 * (col & 3)) * 0x01010101;
        uint32_t c22;
        asm volatile("v_mov_b32 %0, 0x22222222" : "=v"(c22));
        // A load that carries no data but keeps the number of vector-memory operations per
        // step constant (the in-order completion counter is what the ring relies on): four
        // bytes per lane from the zero page into a scratch corner of LDS.
        uint8_t *dummy_dst = lds + LDS_RING_BYTES + LDS_PART_BYTES + 256 + wave * 256;
        const uint32_t *dummy_src = zero_page;

        // ---- sign-tile stream cursor (runs RING_D tiles ahead of the MFMAs)
        int a_op = -1, a_u = 0, a_u1 = 0;
        const uint8_t *a_base = nullptr;
        uint32_t a_count = 0;
        auto issue_a = [&]() {
            while (a_u >= a_u1 && a_op < n_ops) {
                a_op = __builtin_amdgcn_readfirstlane(a_op + 1);
                if (a_op < n_ops) {
                    const int CT = __builtin_amdgcn_readfirstlane(ops[a_op].CT);
                    const Span s = op_span(__builtin_amdgcn_readfirstlane(ops[a_op].RT), CT, grp, G, wave);
                    a_u = s.u0; a_u1 = s.u1;
                    a_base = uniform_ptr(ops[a_op].bits) + (size_t)s.rt0 * CT * 1024;
                }
            }
            uint8_t *slot = ring + (a_count % RING_D) * 1024;
            if (a_u < a_u1) {
                __builtin_amdgcn_global_load_lds(a_base + ((size_t)a_u * 64 + lane) * 16, RB_LDS(slot), 16, 0, 0);
                ++a_u;
            } else {
                __builtin_amdgcn_global_load_lds(dummy_src, RB_LDS(dummy_dst), 4, 0, 0);
            }
            ++a_count;
        };
        auto issue_dummies = [&](int n) {
            for (int i = 0; i < n; ++i) __builtin_amdgcn_global_load_lds(dummy_src, RB_LDS(dummy_dst), 4, 0, 0);
        };

#pragma unroll 1
        for (int d = 0; d < RING_D; ++d) { issue_a(); issue_dummies(4); }
        uint32_t c_count = 0;     // tiles consumed so far (ring slot = c_count % RING_D)
        BTile B[NB];
#pragma unroll
        for (int i = 0; i < NB; ++i)
#pragma unroll
            for (int r = 0; r < 4; ++r) B[i].r[r] = (v4i){0, 0, 0, 0};

        // Operand loads are written as instructions, so the compiler does not know that their
        // target registers stay busy until the data arrives.  Naming the registers here keeps
        // them allocated (never reused as temporaries) across the code between two stages.
        auto keep_operands = [&]() {
#pragma unroll
            for (int i = 0; i < NB; ++i)
                asm volatile("" : "+v"(B[i].r[0]), "+v"(B[i].r[1]), "+v"(B[i].r[2]), "+v"(B[i].r[3]));
        };

        for (int st = 0; st < n_stages; ++st) {
            const Stage stage = stages[st];
            if (stage.wait_before) lds_barrier();        // released by the polling wavefront
            keep_operands();

            // ---- this wavefront's tiles of the stage, op after op
            // B cursor: (op index in stage, tile) -> address of the expanded input
            int b_op = stage.op0 - 1, b_u = 0, b_u1 = 0, b_CT = 1;
            v4i b_rsrc = {0, 0, 0, 0x00020000};               // empty buffer: every load returns zero
            auto issue_b = [&](BTile &dst) {
                while (b_u >= b_u1 && b_op < stage.op0 + stage.nops) {
                    b_op = __builtin_amdgcn_readfirstlane(b_op + 1);
                    if (b_op < stage.op0 + stage.nops) {
                        b_CT = __builtin_amdgcn_readfirstlane(ops[b_op].CT);
                        const Span s = op_span(__builtin_amdgcn_readfirstlane(ops[b_op].RT), b_CT, grp, G, wave);
                        b_u = s.u0; b_u1 = s.u1;
                        const uint64_t up = (uint64_t)uniform_ptr(ops[b_op].up);
                        // raw buffer descriptor: base, stride 0, size of token pair 0, 32-bit untyped
                        b_rsrc[0] = (int)(uint32_t)up;
                        b_rsrc[1] = (int)((uint32_t)(up >> 32) & 0xffffu);
                        b_rsrc[2] = 2 * b_CT * UP_BLOCK_BYTES;
                        b_rsrc[3] = 0x00020000;
                    }
                }
                // Always four loads, written as instructions so that their order and their number
                // per step are exactly what the wait before the MFMAs counts on.  Without a tile
                // left, and in lanes beyond the used operand columns, the offset lies past the end
                // of the buffer: a bounds-checked zero, no memory access.
                const bool valid = b_u < b_u1;
                const int ct = valid ? b_u % b_CT : 0;
                const uint32_t off0 = (valid && col < ncols)
                                          ? (uint32_t)((2 * ct) * UP_BLOCK_BYTES + col * 128 + qd * 32)
                                          : 0x80000000u;
                asm volatile("buffer_load_dwordx4 %0, %4, %5, 0 offen sc1\n\t"
                             "buffer_load_dwordx4 %1, %4, %5, 0 offen offset:16 sc1\n\t"
                             "buffer_load_dwordx4 %2, %4, %5, 0 offen offset:2048 sc1\n\t"
                             "buffer_load_dwordx4 %3, %4, %5, 0 offen offset:2064 sc1"
                             : "=&v"(dst.r[0]), "=&v"(dst.r[1]), "=&v"(dst.r[2]), "=&v"(dst.r[3])
                             : "v"(off0), "s"(b_rsrc)
                             : "memory");
                b_u += valid ? 1 : 0;
            };

            // consume cursor
            int c_op = stage.op0 - 1, c_u = 0, c_u1 = 0, c_CT = 1, slot_base = 0, next_slot_base = 0;
            v4f acc0 = {0, 0, 0, 0}, acc1 = {0, 0, 0, 0};
            const int parity = st & 1;
            auto flush = [&](int slot) {
                float *dstp = part + (size_t)(parity * MAXSLOT + slot) * 512 + (4 * qd) * 16 + col;
                const uint32_t a = lds_addr(dstp);
                asm volatile("ds_add_f32 %0, %1\n\tds_add_f32 %0, %2 offset:64\n\tds_add_f32 %0, %3 offset:128\n\t"
                             "ds_add_f32 %0, %4 offset:192\n\tds_add_f32 %0, %5 offset:1024\n\t"
                             "ds_add_f32 %0, %6 offset:1088\n\tds_add_f32 %0, %7 offset:1152\n\t"
                             "ds_add_f32 %0, %8 offset:1216\n\ts_waitcnt lgkmcnt(0)"
                             :
                             : "v"(a), "v"(acc0[0]), "v"(acc0[1]), "v"(acc0[2]), "v"(acc0[3]), "v"(acc1[0]),
                               "v"(acc1[1]), "v"(acc1[2]), "v"(acc1[3])
                             : "memory");
                acc0 = (v4f){0, 0, 0, 0};
                acc1 = (v4f){0, 0, 0, 0};
            };

#pragma unroll
            for (int i = 0; i < NB; ++i) { issue_b(B[i]); issue_dummies(1); }

            bool more = true;
            while (more) {
#pragma unroll
                for (int s = 0; s < NB; ++s) {
                    // advance the consume cursor to the next tile of this wavefront in the stage
                    while (c_u >= c_u1 && c_op < stage.op0 + stage.nops) {
                        c_op = __builtin_amdgcn_readfirstlane(c_op + 1);
                        slot_base = next_slot_base;
                        if (c_op < stage.op0 + stage.nops) {
                            c_CT = __builtin_amdgcn_readfirstlane(ops[c_op].CT);
                            const Span sp = op_span(__builtin_amdgcn_readfirstlane(ops[c_op].RT), c_CT, grp, G, wave);
                            c_u = sp.u0; c_u1 = sp.u1;
                            next_slot_base = slot_base + sp.nrt;
                        }
                    }
                    if (c_u >= c_u1) { more = false; break; }
                    // Every step issues exactly five vector-memory loads (four operand loads, one
                    // sign tile or its stand-in) and loads complete in order.  The operand of this
                    // tile was requested NB steps ago, followed by 5 * NB - 4 younger loads; the
                    // sign tile is older still (RING_D > NB).  So "at most 5 * NB - 4 outstanding"
                    // means both have arrived.
                    uint4 w;
                    {
                        const uint32_t addr = lds_addr(ring + (c_count % RING_D) * 1024 + lane * 16);
                        asm volatile("s_waitcnt vmcnt(%6)\n\tds_read_b128 %0, %5\n\ts_waitcnt lgkmcnt(0)"
                                     : "=v"(w), "+v"(B[s].r[0]), "+v"(B[s].r[1]), "+v"(B[s].r[2]), "+v"(B[s].r[3])
                                     : "v"(addr), "n"(5 * NB - 4)
                                     : "memory");
                    }
                    ++c_count;
                    const BTile bt = B[s];
                    v8i b0, b1;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        b0[i] = bt.r[0][i]; b0[4 + i] = bt.r[1][i];
                        b1[i] = bt.r[2][i]; b1[4 + i] = bt.r[3][i];
                    }
                    acc0 = mfma_signs(w.x, b0, acc0, c22, scale_b);
                    acc1 = mfma_signs(w.y, b0, acc1, c22, scale_b);
                    acc0 = mfma_signs(w.z, b1, acc0, c22, scale_b);
                    acc1 = mfma_signs(w.w, b1, acc1, c22, scale_b);
                    const int local_rt = c_u / c_CT;
                    ++c_u;
                    if (c_u == c_u1 || c_u % c_CT == 0) flush(slot_base + local_rt);
                    issue_b(B[s]);
                    issue_a();
                }
            }
            lds_barrier();                                    // partial sums of the stage are in LDS
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // nothing may land in LDS after the end
        keep_operands();
    } else {
        // =================== finishing / hand-over wavefront ================
        const int ew = wave - CWAVES;
        uint32_t sig = 0;                                     // signalling stages seen so far
        bool failed = false;                                  // a wait timed out: stop waiting, report
        for (int st = 0; st < n_stages; ++st) {
            const Stage stage = stages[st];
            if (stage.wait_before) {
                // wait until every workgroup has published the previous signalling stage
                if (ew == 0 && !failed) {
                    const uint32_t target = epoch0 + sig - 1u;
                    int spins = 0;
                    while (true) {
                        bool ok = true;
                        for (int i = lane; i < G; i += 64)
                            ok = ok && (int)(__hip_atomic_load(&flags[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) -
                                             target) >= 0;
                        if (__all(ok)) break;
                        if (++spins > (1 << 17)) {
                            if (lane == 0) __hip_atomic_store(error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            failed = true;
                            break;
                        }
                        __builtin_amdgcn_s_sleep(2);
                    }
                }
                lds_barrier();
            }
            lds_barrier();                                    // partial sums complete
            const int parity = st & 1;
            // slots of this workgroup in this stage, dealt round-robin to the four wavefronts
            int slot = 0;
            for (int o = stage.op0; o < stage.op0 + stage.nops; ++o) {
                const Op &op = ops[o];
                const Span sp = op_span(op.RT, op.CT, grp, G, 0);
                for (int r = 0; r < sp.nrt; ++r, ++slot) {
                    if ((slot & (EWAVES - 1)) != ew) continue;
                    float *P = part + (size_t)(parity * MAXSLOT + slot) * 512;
                    const int row = lane & 15, tok = (lane >> 4) & 1;
                    const int grow = (sp.rt0 + r) * 16 + row;
                    float y = 0.f;
                    if (lane < 32) {
#pragma unroll
                        for (int p = 0; p < 2; ++p) {
                            const float4 v = *reinterpret_cast<const float4 *>(P + (p * 16 + row) * 16 + 8 * tok + 4 * p);
                            const float gsc = grow < op.out
                                                  ? __half2float(reinterpret_cast<const __half *>(op.g)[(size_t)p * op.out + grow]) *
                                                        op.inv_sc[p]
                                                  : 0.f;
                            y += gsc * ((v.x + v.y) + (v.z + v.w));
                        }
                    }
                    // clear the slot for its next use
                    reinterpret_cast<float4 *>(P)[lane] = make_float4(0, 0, 0, 0);
                    reinterpret_cast<float4 *>(P)[lane + 64] = make_float4(0, 0, 0, 0);
                    if (lane < 32 && tok < T && grow < op.out) {
                        const __half y16 = __float2half_rn(y);
                        reinterpret_cast<__half *>(op.y)[(size_t)tok * op.out + grow] = y16;
                        const float yf = __half2float(y16);
                        for (int c = 0; c < op.n_cons; ++c) {
                            const Op &m = ops[op.cons[c]];
                            const int CB = col_tiles(m.in) * 2;
#pragma unroll
                            for (int p = 0; p < 2; ++p) {
                                const float h = __half2float(reinterpret_cast<const __half *>(m.h)[(size_t)p * m.in + grow]);
                                const uint32_t terms = expand4(h * yf * m.sc[p]);
#pragma unroll
                                for (int t = 0; t < 4; ++t)
                                    __hip_atomic_store(m.up + up_offset(CB, tok, p, t, grow), (uint8_t)(terms >> (8 * t)),
                                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            }
                        }
                    }
                }
            }
            if (stage.signal_after) {
                // all stores of this wavefront have reached memory, then count in; the last of the
                // four publishes the workgroup's flag
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                uint32_t old = 0;
                if (lane == 0) old = atomicAdd(&misc[0], 1u);
                old = __builtin_amdgcn_readfirstlane(old);
                if (old == (uint32_t)EWAVES * (sig + 1) - 1u && lane == 0)
                    __hip_atomic_store(&flags[grp], epoch0 + sig, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                ++sig;
            }
        }
    }
}

// ------------------------------------------------------------------ host ---
static Layout make_layout(int n_ops, int n_stages, int n_groups, size_t up_total)
{
    Layout L;
    size_t o = sizeof(Header);
    o = align_up(o, 128); L.ops = o; o += sizeof(Op) * (size_t)n_ops;
    o = align_up(o, 128); L.stages = o; o += sizeof(Stage) * (size_t)n_stages;
    o = align_up(o, 128); L.flags = o; o += sizeof(uint32_t) * (size_t)n_groups;
    o = align_up(o, 128); L.error = o; o += 128;
    L.zero = o; o += 128;
    o = align_up(o, 256); L.up = o; o += up_total;
    L.total = align_up(o, 256);
    return L;
}

static int device_groups()
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
    return L->K == 2 && T >= 1 && T <= MAX_T && L->in % 32 == 0;
}

size_t plan_workspace_bytes(const rb_layer *layers, int n_layers, int n_ops, int T)
{
    // upper bound: every op could use the widest layer
    size_t up_max = 0;
    for (int l = 0; l < n_layers; ++l) up_max = std::max(up_max, up_bytes(layers[l].in, T));
    const int G = 1024;   // bound on compute units
    return make_layout(n_ops, n_ops, G, align_up(up_max, 256) * (size_t)n_ops).total;
}

static uint32_t g_epoch = 1;

int run_plan(const rb_layer *layers, const rb_stack_op *sops, int n_ops, uint16_t *const *bufs, int T,
             void *workspace, size_t workspace_bytes_, hipStream_t stream)
{
    const int G = device_groups();
    if (G <= 0) return RB_ERR_HIP;

    // ---- ops, consumers, stages
    std::vector<Op> ops((size_t)n_ops);
    std::vector<int> expand_list;
    size_t up_total = 0;
    std::vector<size_t> up_off((size_t)n_ops);
    for (int n = 0; n < n_ops; ++n) {
        const rb_layer &L = layers[sops[n].layer];
        Op &o = ops[(size_t)n];
        std::memset(&o, 0, sizeof(Op));
        o.bits = static_cast<const uint32_t *>(L.bits);
        o.g = L.g; o.h = L.h;
        o.x = bufs[sops[n].src];
        o.y = bufs[sops[n].dst];
        o.out = L.out; o.in = L.in;
        o.RT = row_tiles(L.out); o.CT = col_tiles(L.in);
        up_off[(size_t)n] = up_total;
        up_total += align_up(up_bytes(L.in, T), 256);
        // producer of this op's input: the last earlier op that writes the same buffer
        int producer = -1;
        for (int m = n - 1; m >= 0; --m)
            if (sops[m].dst == sops[n].src) { producer = m; break; }
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
    std::vector<Stage> stages;
    {
        int op0 = 0;
        while (op0 < n_ops) {
            Stage s{op0, 0, 0, 0};
            int slots = 0;
            for (int n = op0; n < n_ops; ++n) {
                bool conflict = false;
                for (int m = op0; m < n; ++m)
                    if (sops[m].dst == sops[n].src || sops[m].dst == sops[n].dst || sops[m].src == sops[n].dst)
                        conflict = true;
                const int per_group = (ops[(size_t)n].RT + G - 1) / G;
                if (per_group > MAXSLOT) return RB_ERR_UNSUPPORTED;
                if (conflict || slots + per_group > MAXSLOT) break;
                slots += per_group;
                ++s.nops;
            }
            for (int n = s.op0; n < s.op0 + s.nops; ++n)
                if (!ops[(size_t)n].expand_x) s.wait_before = 1;
            stages.push_back(s);
            op0 += s.nops;
        }
        // a stage signals if a later stage waits (the wait of stage s+1.. refers to the latest signal)
        for (size_t s = 0; s + 1 < stages.size(); ++s)
            for (size_t r = s + 1; r < stages.size(); ++r)
                if (stages[r].wait_before) { stages[s].signal_after = 1; break; }
        // every waiting stage must follow a signalling stage that covers all earlier writes:
        // make each stage before a waiting stage signal
        for (size_t s = 1; s < stages.size(); ++s)
            if (stages[s].wait_before) stages[s - 1].signal_after = 1;
    }
    const int n_stages = (int)stages.size();
    int n_signals = 0;
    for (const Stage &s : stages) n_signals += s.signal_after;

    const Layout lay = make_layout(n_ops, n_stages, G, up_total);
    if (workspace_bytes_ < lay.total) return RB_ERR_WORKSPACE;
    uint8_t *ws = static_cast<uint8_t *>(workspace);
    for (int n = 0; n < n_ops; ++n) ops[(size_t)n].up = ws + lay.up + up_off[(size_t)n];

    Header hdr{};
    hdr.n_ops = n_ops; hdr.n_stages = n_stages; hdr.T = T; hdr.n_groups = G;
    hdr.epoch0 = g_epoch;
    g_epoch += (uint32_t)n_signals + 2u;

    // ---- upload (stream-ordered copies from host memory that lives until they are staged)
    static thread_local std::vector<uint8_t> blob;
    blob.assign(lay.up, 0);
    std::memcpy(blob.data(), &hdr, sizeof(hdr));
    std::memcpy(blob.data() + lay.ops, ops.data(), sizeof(Op) * (size_t)n_ops);
    std::memcpy(blob.data() + lay.stages, stages.data(), sizeof(Stage) * (size_t)n_stages);
    std::vector<int> which = expand_list;
    const size_t which_off = lay.error + 64;   // spare bytes after the error word hold the expand list
    if (which.size() * sizeof(int) > 64) {
        // long lists go behind the zero page instead of the spare bytes: not expected for decoder stacks
        return RB_ERR_UNSUPPORTED;
    }
    std::memcpy(blob.data() + which_off, which.data(), which.size() * sizeof(int));
    if (hipMemcpyAsync(ws, blob.data(), lay.flags, hipMemcpyHostToDevice, stream) != hipSuccess) return RB_ERR_HIP;
    if (hipMemcpyAsync(ws + which_off, blob.data() + which_off, 64, hipMemcpyHostToDevice, stream) != hipSuccess)
        return RB_ERR_HIP;

    Header *d_hdr = reinterpret_cast<Header *>(ws);
    Op *d_ops = reinterpret_cast<Op *>(ws + lay.ops);
    Stage *d_stages = reinterpret_cast<Stage *>(ws + lay.stages);
    uint32_t *d_flags = reinterpret_cast<uint32_t *>(ws + lay.flags);
    uint32_t *d_error = reinterpret_cast<uint32_t *>(ws + lay.error);
    uint32_t *d_zero = reinterpret_cast<uint32_t *>(ws + lay.zero);
    const int *d_which = reinterpret_cast<const int *>(ws + which_off);

    hipLaunchKernelGGL(prep_kernel, dim3(n_ops), dim3(256), 0, stream, d_hdr, d_ops, d_flags, d_error, d_zero, 1);
    if (!expand_list.empty()) {
        int max_in = 0;
        for (int n : expand_list) max_in = std::max(max_in, ops[(size_t)n].in);
        hipLaunchKernelGGL(expand_kernel, dim3((max_in + 255) / 256, T, (unsigned)expand_list.size()), dim3(256), 0,
                           stream, d_hdr, d_ops, d_which);
    }
    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(stack_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES) != hipSuccess)
            return RB_ERR_HIP;
        attr_set = true;
    }
    hipLaunchKernelGGL(stack_kernel, dim3(G), dim3(THREADS), LDS_BYTES, stream, d_hdr, d_ops, d_stages, d_flags,
                       d_error, d_zero);
    return hipGetLastError() == hipSuccess ? RB_OK : RB_ERR_HIP;
}

}  // namespace mx
}  // namespace rb
