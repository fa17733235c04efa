// Matrix-core decode path: set-up kernels, the persistent kernel that runs a whole list of ops in
// one launch, and its host planner.  See rb_mx.h for the arithmetic, the operand layout and the
// plan structures.
//
// The plan is a list of phases; a phase is a range of row tiles of one op, dealt to the workgroups
// (one per compute unit) in contiguous shares.  Every workgroup walks the phases in order, and no
// barrier separates them.  Inside a workgroup three kinds of wavefronts work side by side:
//   * loading wavefronts stream the workgroup's sign tiles, in plan order, from HBM into a ring of
//     128 tiles in LDS (global_load_lds, non-temporal).  The weights do not depend on activations,
//     so this stream never waits for another compute unit: it runs as far ahead as the ring
//     allows, across ops, and keeps HBM busy while the rest of the workgroup waits for inputs.
//     Keeping these loads on wavefronts of their own matters because vector-memory loads of one
//     wavefront complete in order: a consumer that also prefetched weights would find its (short)
//     operand loads queued behind (long) weight loads.
//   * consuming wavefronts take the tiles of a phase in units of (row tile, chunk of column tiles),
//     read the matching part of the expanded input from memory (L2), expand the signs to fp4 and
//     issue four matrix instructions per tile (Section 4.1: the signed accumulation), and leave one
//     partial sum per unit in LDS.
//   * finishing wavefronts add the partial sums of a row in chunk order, form y = sum_k g_k * acc_k
//     (Eq. stacked binary weight), round to fp16 once, store, and write h (.) y as four bf8 terms
//     into the expanded input of every op that reads y (the input scaling of Section 4.1, done
//     once by the producer) with device-scope 16-byte stores.
// Wavefronts of a workgroup meet through counters in LDS (tiles landed, phases done), never through
// a barrier, and every wait is bounded: when one runs out the workgroup stops waiting, finishes
// with meaningless outputs and leaves a mark for rb_stack_status.
//
// Hand-over between compute units: before a launch every 16-byte group of an expanded input that
// an op of the launch will write is filled with 0xff bytes, which no bf8 term has.  Producers
// just store.  A consumer starts on a dependent phase once its own workgroup has finished the
// producing phase and a pause has passed (the other workgroups finish at about the same time),
// reads operand tiles with plain loads (shared by the 32 compute units of an XCD through its L2)
// and checks every 32-bit word it got: a tile with a word that still reads 0xffffffff was fetched
// before its producer's store had landed and is read again past the L2 until it is complete.
// The pause is a matter of speed, not of correctness.  The check does not assume that a 16-byte
// store becomes visible as a whole, only that an aligned 32-bit word does.
//
// The order of the phases is the planner's: ops on the longest dependency chain go first, and ops
// that nobody waits for (or not soon) are placed behind them, where they fill the time a
// hand-over takes.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <map>
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
// Pointers read from a table are generic; dereferencing them as such makes FLAT instructions,
// which also count as LDS traffic.  They are cast to the global address space.
#define RB_GLOBAL(T, p) ((__attribute__((address_space(1))) T *)(p))

constexpr int SPIN_LIMIT = 1 << 20;        // polls of a bounded wait before it gives up
constexpr int CACHE_NT = 2;                // non-temporal: every sign tile is read once

// ---------------------------------------------------------------- helpers ---
__device__ __forceinline__ uint32_t lds_addr(const void *p) { return (uint32_t)(size_t)RB_LDS(p); }

// Control words in LDS are read and written with explicit instructions: the compiler then neither
// caches them nor ties them to the asynchronous global->LDS copies of the loading wavefronts.
__device__ __forceinline__ uint32_t ctrl_read(uint32_t addr)
{
    uint32_t v;
    asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(addr) : "memory");
    return (uint32_t)__builtin_amdgcn_readfirstlane((int)v);
}
__device__ __forceinline__ void ctrl_write(uint32_t addr, uint32_t v)
{
    asm volatile("ds_write_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : : "v"(addr), "v"(v) : "memory");
}
__device__ __forceinline__ void ctrl_add(uint32_t addr, uint32_t v)
{
    asm volatile("ds_add_u32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : : "v"(addr), "v"(v) : "memory");
}
__device__ __forceinline__ uint32_t clock32() { return (uint32_t)__builtin_amdgcn_s_memtime(); }

// Bounded waits on control words, as a few scalar instructions each: polls the word at `addr` (the
// smaller of the two words at `addr` for wait_pair) until it is at least `need` or `limit` polls
// have passed, and returns what it read last (less than `need`: the wait ran out).
__device__ __forceinline__ uint32_t wait_word(uint32_t addr, uint32_t need, uint32_t limit)
{
    uint32_t val, left, tmp;
    need = (uint32_t)__builtin_amdgcn_readfirstlane((int)need);       // both are the same in every lane
    limit = (uint32_t)__builtin_amdgcn_readfirstlane((int)limit);
    asm volatile("s_mov_b32 %[left], %[limit]\n"
                 "1:\n\t"
                 "ds_read_b32 %[tmp], %[addr]\n\t"
                 "s_waitcnt lgkmcnt(0)\n\t"
                 "v_readfirstlane_b32 %[val], %[tmp]\n\t"
                 "s_cmp_ge_u32 %[val], %[need]\n\t"
                 "s_cbranch_scc1 2f\n\t"
                 "s_sleep 1\n\t"
                 "s_sub_u32 %[left], %[left], 1\n\t"
                 "s_cmp_lg_u32 %[left], 0\n\t"
                 "s_cbranch_scc1 1b\n"
                 "2:"
                 : [val] "=&s"(val), [left] "=&s"(left), [tmp] "=&v"(tmp)
                 : [addr] "v"(addr), [need] "s"(need), [limit] "s"(limit)
                 : "scc", "memory");
    return val;
}
__device__ __forceinline__ uint32_t wait_pair(uint32_t addr, uint32_t need, uint32_t limit)
{
    uint32_t val, other, left, tmp0, tmp1;
    need = (uint32_t)__builtin_amdgcn_readfirstlane((int)need);
    limit = (uint32_t)__builtin_amdgcn_readfirstlane((int)limit);
    asm volatile("s_mov_b32 %[left], %[limit]\n"
                 "1:\n\t"
                 "ds_read_b32 %[tmp0], %[addr]\n\t"
                 "ds_read_b32 %[tmp1], %[addr] offset:4\n\t"
                 "s_waitcnt lgkmcnt(0)\n\t"
                 "v_readfirstlane_b32 %[val], %[tmp0]\n\t"
                 "v_readfirstlane_b32 %[other], %[tmp1]\n\t"
                 "s_min_u32 %[val], %[val], %[other]\n\t"
                 "s_cmp_ge_u32 %[val], %[need]\n\t"
                 "s_cbranch_scc1 2f\n\t"
                 "s_sleep 1\n\t"
                 "s_sub_u32 %[left], %[left], 1\n\t"
                 "s_cmp_lg_u32 %[left], 0\n\t"
                 "s_cbranch_scc1 1b\n"
                 "2:"
                 : [val] "=&s"(val), [other] "=&s"(other), [left] "=&s"(left), [tmp0] "=&v"(tmp0), [tmp1] "=&v"(tmp1)
                 : [addr] "v"(addr), [need] "s"(need), [limit] "s"(limit)
                 : "scc", "memory");
    return val;
}

// "at most N vector-memory operations outstanding" (vmcnt in bits 3:0 and 15:14 of the immediate)
template <int N> __device__ __forceinline__ void wait_vm()
{
    static_assert(N >= 0 && N < 64, "vmcnt has six bits");
    __builtin_amdgcn_s_waitcnt((N & 0xf) | ((N >> 4) << 14) | (0x7 << 4) | (0xf << 8));
}

// ------------------------------------------------------------ prep kernel ---
// One workgroup per op: power-of-two scale of each path's input scales and the zero fill of the
// expanded-input array (padding columns and unused operand columns must read as zero).
__global__ __launch_bounds__(256) void prep_kernel(const Header *hdr, Op *ops, uint32_t *error)
{
    const int o = blockIdx.x;
    Op &op = ops[o];
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
            const float sc = input_scale(red[0]);
            op.sc[p] = sc;
            op.inv_sc[p] = 1.f / sc;
        }
        __syncthreads();
    }
    const size_t n16 = up_bytes(op.in, hdr->T) / 16;
    uint4 *up = reinterpret_cast<uint4 *>(op.up);
    for (size_t i = threadIdx.x; i < n16; i += 256) up[i] = make_uint4(0, 0, 0, 0);
    if (o == 0 && threadIdx.x < 2) error[threadIdx.x] = 0;      // the give-up mark and the count of tiles read again
}

// Second set-up pass (needs the scales of every op): the phase records and the shares of every
// workgroup.  One workgroup per phase.
__global__ __launch_bounds__(256) void phase_kernel(const Header *hdr, const Op *ops, const PhaseSeed *seeds,
                                                    Phase *phases, Share *shares)
{
    const int p = blockIdx.x, G = hdr->n_groups, T = hdr->T;
    const PhaseSeed sd = seeds[p];
    const Op &op = ops[sd.op];
    if (threadIdx.x == 0) {
        Phase ph;
        memset(&ph, 0, sizeof(ph));
        ph.bits = (uint64_t)op.bits;
        ph.up = (uint64_t)op.up;
        ph.y = (uint64_t)op.y;
        ph.g = (uint64_t)op.g;
        ph.out = op.out; ph.CT = op.CT; ph.rt_first = sd.rt_first; ph.n_rt = sd.n_rt;
        ph.dep_phase = op.dep >= 0 ? ops[op.dep].last_phase : -1;
        ph.n_cons = op.n_cons;
        ph.inv_sc[0] = op.inv_sc[0]; ph.inv_sc[1] = op.inv_sc[1];
        ph.chunk = chunk_tiles(op.CT); ph.n_chunks = chunks_of(op.CT);
        ph.up_bytes = (int)up_bytes(op.in, T);
        ph.op = sd.op;
        for (int c = 0; c < op.n_cons; ++c) {
            const Op &m = ops[op.cons[c]];
            ph.cons[c].up = (uint64_t)m.up;
            ph.cons[c].h = (uint64_t)m.h;
            ph.cons[c].sc[0] = m.sc[0]; ph.cons[c].sc[1] = m.sc[1];
            ph.cons[c].in = m.in;
        }
        phases[p] = ph;
    }
    for (int grp = threadIdx.x; grp < G; grp += 256) {
        uint32_t first, count;
        share_rows((uint32_t)sd.n_rt, (uint32_t)((grp + G - sd.rot % G) % G), (uint32_t)G, first, count);
        shares[(size_t)p * G + grp] = Share{sd.rt_first + (int)first, (int)count};
    }
}

// Third set-up pass: the unit lists of the consuming wavefronts (see Unit).  One thread per
// (workgroup, consuming wavefront) walks the phases.
__global__ __launch_bounds__(64) void unit_kernel(const Header *hdr, const Phase *phases, const Share *shares,
                                                  const uint8_t *up_base, Unit *units)
{
    const int G = hdr->n_groups, T = hdr->T, stride = hdr->unit_stride;
    const int id = blockIdx.x * 64 + threadIdx.x;
    if (id >= G * NC) return;
    const int grp = id / NC, c = id % NC;
    Unit *list = units + (size_t)id * stride;
    uint32_t S = 0;                               // tiles of the workgroup's sequence before this phase
    int e = 0;
    for (int p = 0; p < hdr->n_phases; ++p) {
        const Phase &ph = phases[p];
        const Share sh = shares[(size_t)p * G + grp];
        const int U = sh.nrt * ph.n_chunks;
        const int ub = c * U / NC, ue = (c + 1) * U / NC;
        for (int u = ub; u < ue && e < stride - 65; ++u) {
            const int slot = u / ph.n_chunks, chunk = u % ph.n_chunks;
            const int ct0 = chunk * ph.chunk, ct1 = min(ph.CT, ct0 + ph.chunk);
            Unit un;
            un.seq0 = S + (uint32_t)(slot * ph.CT + ct0);
            un.up_off = (uint32_t)((const uint8_t *)ph.up - up_base) + (uint32_t)ct0 * (uint32_t)(2 * up_block_bytes(T));
            un.w2 = (uint32_t)(ct1 - ct0) | (uint32_t)(((p % NPAR) * MAX_SLOTS + slot) * MAX_CHUNKS + chunk) << UNIT_PART_SHIFT |
                    (u == ue - 1 ? UNIT_LAST : 0u);
            un.w3 = (uint32_t)p | (uint32_t)(ph.dep_phase + 1) << 16;
            list[e++] = un;
        }
        S += (uint32_t)(sh.nrt * ph.CT);
    }
    for (; e < stride; ++e) list[e] = Unit{0u, 0u, 0u, 0u};      // the end mark (and what is read ahead of it)
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
    const int T = hdr->T;
    const float x = __half2float(reinterpret_cast<const __half *>(op.x)[(size_t)tok * op.in + j]);
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const float h = __half2float(reinterpret_cast<const __half *>(op.h)[(size_t)p * op.in + j]);
        const uint32_t terms = expand4(h * x * op.sc[p]);
#pragma unroll
        for (int t = 0; t < 4; ++t) op.up[up_offset(T, tok, p, t, j)] = (uint8_t)(terms >> (8 * t));
    }
}

// Before every launch: the expanded input of every op that a producer of this launch will write
// is set to "not written yet" (0xff in every byte of the 16-byte groups of real columns: no bf8
// term is 0xff; padding columns read as zero).  POISON_SPLIT workgroups per op.
constexpr int POISON_SPLIT = 4;
__global__ __launch_bounds__(256) void poison_kernel(const Op *ops, int T)
{
    const Op &op = ops[blockIdx.x];
    if (op.dep < 0) return;
    const int groups = (int)(up_bytes(op.in, T) / 16);
    uint4 *up = reinterpret_cast<uint4 *>(op.up);
    for (int i = blockIdx.y * 256 + threadIdx.x; i < groups; i += 256 * POISON_SPLIT) {
        // which 16 input columns group i holds (see up_group_offset): a block of 128 columns is
        // [q][half j][operand column 0..7] for one token and [half j][q][operand column 0..15] for two
        const int b = T == 1 ? i >> 6 : i >> 7;
        const int q = (i >> 4) & 3;
        const int j = T == 1 ? (i >> 3) & 1 : (i >> 6) & 1;
        const uint32_t v = b * 128 + j * 64 + q * 16 < op.in ? 0xffffffffu : 0u;
        up[i] = make_uint4(v, v, v, v);
    }
}

// ------------------------------------------------------- persistent kernel ---
template <int TT> struct BTile { v4i r[kop_of(TT)]; };   // operand of one tile: two 128-column blocks

template <int TT>
__global__ __launch_bounds__(THREADS, 1) void chain_kernel(const Phase *__restrict__ phases,
                                                           const Share *__restrict__ shares,
                                                           const Unit *__restrict__ units, int unit_stride,
                                                           const uint8_t *__restrict__ up_base, uint32_t up_total,
                                                           int n_phases, uint32_t *__restrict__ error, int pause_clks)
{
    using Lds = LdsMap<TT>;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int grp = blockIdx.x, G = gridDim.x;
    const uint32_t ctrl = lds_addr(lds + Lds::CTRL_OFF);
    constexpr int KOP = kop_of(TT), NB = nb_of(TT);

    if (threadIdx.x < Lds::CTRL_BYTES / 4) reinterpret_cast<uint32_t *>(lds + Lds::CTRL_OFF)[threadIdx.x] = 0u;
    __syncthreads();

    // a bounded wait ran out: tell the workgroup and the host
    auto give_up = [&]() {
        if (lane == 0) {
            ctrl_write(ctrl + 4 * CTRL_FAILED, 1u);
            __hip_atomic_store(RB_GLOBAL(uint32_t, error), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    };

    if (wave < NL) {
        // ========================= loading wavefront ========================
        // Tile number s of the workgroup's sequence goes to ring slot s mod RING_TILES and is
        // loaded by wavefront s mod NL; a slot may be reused once the phase its former tile
        // belonged to is complete (CTRL_CONSUMED).
        const uint32_t my_landed = ctrl + 4 * (CTRL_LANDED + wave);
        uint32_t S = 0, issued = 0, published = 0, consumed = 0;
        bool failed = false;
        auto publish = [&](uint32_t n) {
            if (lane == 0) ctrl_write(my_landed, n);
            published = n;
        };
        // what the wavefront needs to know about a phase is requested one phase ahead (scalar loads)
        struct Extent { const uint8_t *base; uint32_t n; };
        auto fetch = [&](int p) -> Extent {
            p = min(p, n_phases - 1);
            const Phase *ph = phases + p;
            const Share sh = shares[(size_t)p * G + grp];
            const uint32_t CT = (uint32_t)ph->CT;
            return Extent{reinterpret_cast<const uint8_t *>(ph->bits) + ((size_t)sh.rt0 * CT) * 1024, (uint32_t)sh.nrt * CT};
        };
        Extent nxt = fetch(0);
        for (int p = 0; p < n_phases; ++p) {
            const Extent cur = nxt;
            nxt = fetch(p + 1);
            const uint32_t n = cur.n;
            const uint8_t *base = cur.base + lane * 16;
            for (uint32_t i = ((uint32_t)wave + NL - S % NL) % NL; i < n; i += NL) {
                const uint32_t s = S + i;
                if (s >= consumed + RING_TILES && !failed) {
                    // No free slot.  While waiting for one, announce what lands, a few tiles at a
                    // time, so that this wavefront is never held up by more than eight loads when
                    // a slot becomes free (the consumers may be waiting for exactly these tiles).
                    int spins = 0;
                    for (;;) {
                        consumed = ctrl_read(ctrl + 4 * CTRL_CONSUMED);
                        if (s < consumed + RING_TILES) break;
                        const uint32_t pending = issued - published;
                        if (pending > 40 && LOADER_WINDOW > 40) { wait_vm<40>(); publish(issued - 40); }
                        else if (pending > 32 && LOADER_WINDOW > 32) { wait_vm<32>(); publish(issued - 32); }
                        else if (pending > 24 && LOADER_WINDOW > 24) { wait_vm<24>(); publish(issued - 24); }
                        else if (pending > 16 && LOADER_WINDOW > 16) { wait_vm<16>(); publish(issued - 16); }
                        else if (pending > 8) { wait_vm<8>(); publish(issued - 8); }
                        else if (pending > 4) { wait_vm<4>(); publish(issued - 4); }
                        else if (pending > 0) { wait_vm<0>(); publish(issued); }
                        else {
                            if (ctrl_read(ctrl + 4 * CTRL_FAILED) != 0u) { failed = true; break; }
                            if (++spins > SPIN_LIMIT) { give_up(); failed = true; break; }
                            __builtin_amdgcn_s_sleep(1);
                        }
                    }
                }
                __builtin_amdgcn_global_load_lds(base + (size_t)i * 1024,
                                                 RB_LDS(lds + Lds::RING_OFF + (s % RING_TILES) * 1024), 16, 0, CACHE_NT);
                ++issued;
                if (issued - published > (uint32_t)LOADER_WINDOW) {
                    wait_vm<LOADER_WINDOW>();                 // loads complete in order
                    publish(issued - LOADER_WINDOW);
                }
            }
            S += n;
        }
        wait_vm<0>();
        publish(issued);
    } else if (wave < NL + NC) {
        // ======================== consuming wavefront =======================
        // Walks the list of its units (see Unit).  Operand tiles are requested NB tiles ahead of
        // their use, across units and phases; B[] is the ring they arrive in, and every step of the
        // loop below consumes the tile of ring slot s and requests another into it, so that the
        // number of loads in flight is the same at every use and "at most (NB - 1) * KOP loads
        // outstanding" always means the tile at hand has arrived (loads complete in order).
        const int c = wave - NL;
        const int col = lane & 15, qd = lane >> 4, quad = col >> 2;
        const int scale_b = term_scale(col);
        const uint32_t lane_off = (uint32_t)lane * 16u;
        const uint32_t ring = lds_addr(lds + Lds::RING_OFF);
        uint32_t c22;
        asm volatile("v_mov_b32 %0, 0x22222222" : "=v"(c22));
        // where this lane's partial sums go inside a unit's entry: the first lane of a quad of
        // operand columns holds rows 4 qd .. 4 qd + 3 of (path = quad & 1, token = quad >> 1)
        const uint32_t part_lane = lds_addr(lds + Lds::PART_OFF) + (uint32_t)(((quad & 1) * TT + (quad >> 1)) * 16 + 4 * qd) * 4u;
        const bool part_writer = (col & 3) == 0 && (quad >> 1) < TT;
        constexpr uint32_t TILE_UP = 2 * up_block_bytes(TT);      // bytes of expanded input per sign tile

        // The list is read 64 records at a time with vector loads, a record per lane, and a record
        // is picked out of the registers when a cursor gets to it.  (Scalar loads would be the
        // natural choice for data every lane shares, but they share their completion counter with
        // LDS reads: every LDS access of this loop would wait for a record on its way from HBM.)
        const uint4 *list = reinterpret_cast<const uint4 *>(units + ((size_t)grp * NC + c) * (size_t)unit_stride) + lane;
        // (These loads, too, are written as instructions: the compiler would wait for everything in
        // flight whenever a record is picked.  A block is requested 64 units before its first use,
        // and the waits of the steps in between see to it that it has arrived.  The registers of the
        // block on its way are named by in-out operands only, and the move from "next" to "current"
        // happens inside the statement that requests the block after, so that the compiler never
        // has a reason to copy a register whose load is still in flight.)
        uint32_t a0 = 0, a1 = 0, a2 = 0, a3 = 0;             // records blk0 .. blk0 + 63, one per lane, field by field
        uint32_t b0_ = 0, b1_ = 0, b2_ = 0, b3_ = 0;         // the 64 records after them
        asm volatile("global_load_dword %0, %8, off\n\t"
                     "global_load_dword %1, %8, off offset:4\n\t"
                     "global_load_dword %2, %8, off offset:8\n\t"
                     "global_load_dword %3, %8, off offset:12\n\t"
                     "global_load_dword %4, %8, off offset:1024\n\t"
                     "global_load_dword %5, %8, off offset:1028\n\t"
                     "global_load_dword %6, %8, off offset:1032\n\t"
                     "global_load_dword %7, %8, off offset:1036\n\t"
                     "s_waitcnt vmcnt(0)"
                     : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3), "+v"(b0_), "+v"(b1_), "+v"(b2_), "+v"(b3_)
                     : "v"(list)
                     : "memory");
        uint32_t blk0 = 0;
        auto next_block = [&]() {                             // current <- next, next <- the block after (requested)
            blk0 += 64u;
            asm volatile("v_mov_b32 %0, %4\n\t"
                         "v_mov_b32 %1, %5\n\t"
                         "v_mov_b32 %2, %6\n\t"
                         "v_mov_b32 %3, %7\n\t"
                         "global_load_dword %4, %8, off\n\t"
                         "global_load_dword %5, %8, off offset:4\n\t"
                         "global_load_dword %6, %8, off offset:8\n\t"
                         "global_load_dword %7, %8, off offset:12"
                         : "=&v"(a0), "=&v"(a1), "=&v"(a2), "=&v"(a3), "+v"(b0_), "+v"(b1_), "+v"(b2_), "+v"(b3_)
                         : "v"(list + (blk0 + 64u))
                         : "memory");
        };
        auto unit_at = [&](uint32_t idx) -> Unit {            // blk0 <= idx < blk0 + 128
            const bool in_a = idx - blk0 < 64u;
            const int l = (int)(idx & 63u);
            Unit u;
            u.seq0 = (uint32_t)__builtin_amdgcn_readlane((int)(in_a ? a0 : b0_), l);
            u.up_off = (uint32_t)__builtin_amdgcn_readlane((int)(in_a ? a1 : b1_), l);
            u.w2 = (uint32_t)__builtin_amdgcn_readlane((int)(in_a ? a2 : b2_), l);
            u.w3 = (uint32_t)__builtin_amdgcn_readlane((int)(in_a ? a3 : b3_), l);
            return u;
        };

        uint32_t limit = SPIN_LIMIT;                          // polls a wait may take; 1 once a wait has run out
        uint32_t landed0 = 0, landed1 = 0;                    // what the loading wavefronts announced (cached)
        uint32_t fin_seen = 0;                                // phases all finishing wavefronts have completed (cached)
        auto ran_out = [&]() {
            limit = 1;
            give_up();
        };
        auto wait_finished = [&](uint32_t n) {                // until phases 0 .. n - 1 are finished in this workgroup
            if (fin_seen < n) {
                fin_seen = wait_pair(ctrl + 4 * CTRL_FIN, n, limit);
                if (fin_seen < n) ran_out();
            }
        };
        auto wait_landed = [&](uint32_t s) {                  // until tile s of the sequence is in the ring
            const uint32_t need = s / NL + 1;
            if (s % NL) {
                if (landed1 < need) { landed1 = wait_word(ctrl + 4 * (CTRL_LANDED + 1), need, limit); if (landed1 < need) ran_out(); }
            } else {
                if (landed0 < need) { landed0 = wait_word(ctrl + 4 * CTRL_LANDED, need, limit); if (landed0 < need) ran_out(); }
            }
        };
        // the input of a unit of phase p is complete once phase `need - 1` is finished everywhere:
        // it is here, and the pause has passed (see the head of this file)
        auto pause_left = [&](uint32_t need, uint32_t p) -> bool {
            if (p - (need - 1u) >= 8u) return false;          // long ago: its time stamp is gone
            const uint32_t t0 = ctrl_read(ctrl + 4 * (CTRL_FIN_TIME + ((need - 1u) & 7u)));
            return clock32() - t0 < (uint32_t)pause_clks;
        };
        auto input_ready = [&](uint32_t need, uint32_t p) -> bool {      // without waiting
            if (fin_seen < need) fin_seen = wait_pair(ctrl + 4 * CTRL_FIN, need, 1u);
            return fin_seen >= need && !pause_left(need, p);
        };
        auto wait_input = [&](uint32_t need, uint32_t p) {
            wait_finished(need);
            int spins = 0;
            while (pause_left(need, p) && ++spins < 4096) __builtin_amdgcn_s_sleep(1);
        };

        // ---- the two cursors over the list
        uint32_t ci = 0, c_tile = 0;                          // consuming: unit, tile inside it
        Unit cu = unit_at(0);
        uint32_t ii = 0, i_tile = 0;                          // requesting operands: at most NB units further on
        Unit iu = cu;
        bool stalled = false;                                 // the next unit's input was not complete when its turn came
        BTile<TT> B[NB];
#pragma unroll
        for (int i = 0; i < NB; ++i)
#pragma unroll
            for (int r = 0; r < KOP; ++r) B[i].r[r] = (v4i){0, 0, 0, 0};
        uint32_t soff[NB];                                    // where each requested operand tile lives
        bool stale[NB];                                       // requested while stalled: nothing was read
        // Operand loads are written as instructions and waited for by count (see above): the
        // compiler would wait for every load in flight before each use, which is what the ring is
        // there to avoid.  It therefore cannot know that a ring register is busy until its load
        // lands, so the registers of the ring are only ever named as in-out operands of such
        // statements - requests, the wait, keep_ring() - and stay allocated to the ring throughout.
        // raw buffer descriptor of the plan's expanded inputs: base, stride 0, size, 32-bit untyped
        v4i rs_live;
        rs_live[0] = (int)(uint32_t)(uintptr_t)up_base;
        rs_live[1] = (int)((uint32_t)((uintptr_t)up_base >> 32) & 0xffffu);
        rs_live[2] = (int)up_total;
        rs_live[3] = 0x00020000;
        auto request = [&](BTile<TT> &dst, uint32_t so, bool live) {
            // a buffer of no size (nothing to request) returns zeros without touching memory
            v4i rs = rs_live;
            rs[2] = live ? rs_live[2] : 0;
            if constexpr (TT == 1)
                asm volatile("buffer_load_dwordx4 %0, %2, %3, %4 offen\n\t"
                             "buffer_load_dwordx4 %1, %2, %3, %4 offen offset:1024"
                             : "+v"(dst.r[0]), "+v"(dst.r[1])
                             : "v"(lane_off), "s"(rs), "s"(so)
                             : "memory");
            else
                asm volatile("buffer_load_dwordx4 %0, %4, %5, %6 offen\n\t"
                             "buffer_load_dwordx4 %1, %4, %5, %6 offen offset:1024\n\t"
                             "buffer_load_dwordx4 %2, %4, %5, %6 offen offset:2048\n\t"
                             "buffer_load_dwordx4 %3, %4, %5, %6 offen offset:3072"
                             : "+v"(dst.r[0]), "+v"(dst.r[1]), "+v"(dst.r[2 % KOP]), "+v"(dst.r[3 % KOP])
                             : "v"(lane_off), "s"(rs), "s"(so)
                             : "memory");
        };
        auto keep_ring = [&]() {
#pragma unroll
            for (int i = 0; i < NB; ++i)
#pragma unroll
                for (int r = 0; r < KOP; ++r) asm volatile("" : "+v"(B[i].r[r]));
            asm volatile("" : "+v"(b0_), "+v"(b1_), "+v"(b2_), "+v"(b3_));
        };
        auto issue = [&](BTile<TT> &dst, uint32_t &so, bool &st) {
            bool live = !stalled && (iu.w2 & 0xffu) != 0u;
            if (live && i_tile == 0u) {
                const uint32_t need = iu.w3 >> 16;
                if (need != 0u && !input_ready(need, iu.w3 & 0xffffu)) {
                    stalled = true;                           // stays so until the consumer gets here and waits
                    live = false;
                }
            }
            st = stalled;
            so = (uint32_t)__builtin_amdgcn_readfirstlane((int)(iu.up_off + i_tile * TILE_UP));
            request(dst, so, live);
            if (live && ++i_tile == (iu.w2 & 0xffu)) {
                i_tile = 0u;
                ++ii;
                iu = unit_at(ii);
            }
        };
        auto unwritten = [&](const BTile<TT> &b) -> bool {
            uint32_t m = 0;
#pragma unroll
            for (int r = 0; r < KOP; ++r)
#pragma unroll
                for (int i = 0; i < 4; ++i) m = max(m, (uint32_t)b.r[r][i]);
            return m == 0xffffffffu;
        };
#pragma unroll
        for (int i = 0; i < NB; ++i) issue(B[i], soff[i], stale[i]);

        v4f acc0 = {0, 0, 0, 0}, acc1 = {0, 0, 0, 0};
        bool more = true;
        while (more) {
            keep_ring();
#pragma unroll
            for (int s = 0; s < NB; ++s) {
                const uint32_t n_tiles = cu.w2 & 0xffu;
                if (n_tiles == 0u) { more = false; break; }   // the end mark
                const uint32_t p = cu.w3 & 0xffffu, need = cu.w3 >> 16;
                // Phase p - NPAR must be finished before anything of phase p is filed: its partial
                // sums share LDS with this phase's, and the count of wavefronts that are through
                // with a phase is kept per parity.
                if (c_tile == 0u && p >= (uint32_t)NPAR) wait_finished(p - NPAR + 1u);
                if (stale[s]) {
                    // the request cursor stopped at this very tile: wait for the input, then request
                    // this tile and the NB - 1 after it
                    wait_input(need, p);
                    stalled = false;
#pragma unroll
                    for (int k = 0; k < NB; ++k) issue(B[(s + k) % NB], soff[(s + k) % NB], stale[(s + k) % NB]);
                }
                const uint32_t seq = cu.seq0 + c_tile;
                wait_landed(seq);
                v4u w;
                asm volatile("ds_read_b128 %0, %1\n\ts_waitcnt lgkmcnt(0)"
                             : "=v"(w)
                             : "v"(ring + (seq % RING_TILES) * 1024u + lane_off)
                             : "memory");
                // this tile's operand was requested NB tiles ago, with (NB - 1) * KOP loads after it
                asm volatile("s_waitcnt vmcnt(%0)" : : "n"((NB - 1) * KOP) : "memory");
#pragma unroll
                for (int r = 0; r < KOP; ++r) asm volatile("" : "+v"(B[s].r[r]));
                if (need != 0u && limit > 1u && __ballot(unwritten(B[s])) != 0ull) {
                    // Requested before its producer's stores had landed (or this XCD's L2 got hold of
                    // the lines early): read the tile again past the L2 until every word of it has
                    // been written.  Nothing may be in flight while the compiler can see a loop.
                    asm volatile("s_waitcnt vmcnt(0)" : : : "memory");
                    keep_ring();
                    int tries = 0;
                    do {
                        __builtin_amdgcn_s_sleep(4);
                        if constexpr (TT == 1)
                            asm volatile("buffer_load_dwordx4 %0, %2, %3, %4 offen sc1\n\t"
                                         "buffer_load_dwordx4 %1, %2, %3, %4 offen offset:1024 sc1\n\t"
                                         "s_waitcnt vmcnt(0)"
                                         : "+v"(B[s].r[0]), "+v"(B[s].r[1])
                                         : "v"(lane_off), "s"(rs_live), "s"(soff[s])
                                         : "memory");
                        else
                            asm volatile("buffer_load_dwordx4 %0, %4, %5, %6 offen sc1\n\t"
                                         "buffer_load_dwordx4 %1, %4, %5, %6 offen offset:1024 sc1\n\t"
                                         "buffer_load_dwordx4 %2, %4, %5, %6 offen offset:2048 sc1\n\t"
                                         "buffer_load_dwordx4 %3, %4, %5, %6 offen offset:3072 sc1\n\t"
                                         "s_waitcnt vmcnt(0)"
                                         : "+v"(B[s].r[0]), "+v"(B[s].r[1]), "+v"(B[s].r[2 % KOP]), "+v"(B[s].r[3 % KOP])
                                         : "v"(lane_off), "s"(rs_live), "s"(soff[s])
                                         : "memory");
                    } while (__ballot(unwritten(B[s])) != 0ull && ++tries < (1 << 16));
                    if (lane == 0) ctrl_add(ctrl + 4 * CTRL_WAITED, 1u);
                    if (tries >= (1 << 16)) ran_out();
                    // (everything requested so far has landed now, so the waits of the next steps hold)
                }
                v8i b0, b1;
                if constexpr (TT == 1) {
                    // lanes 0..7 of a row of 16 hold the first four registers of their column; the
                    // other four sit eight lanes further on (row_shl:8).  Lanes 8..15 end up with
                    // bytes of no meaning: their columns of the product are never read.
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        b0[i] = B[s].r[0][i];
                        b0[4 + i] = __builtin_amdgcn_update_dpp(0, B[s].r[0][i], 0x108, 0xf, 0xf, true);
                        b1[i] = B[s].r[1][i];
                        b1[4 + i] = __builtin_amdgcn_update_dpp(0, B[s].r[1][i], 0x108, 0xf, 0xf, true);
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        b0[i] = B[s].r[0][i]; b0[4 + i] = B[s].r[1][i];
                        b1[i] = B[s].r[2 % KOP][i]; b1[4 + i] = B[s].r[3 % KOP][i];
                    }
                }
                acc0 = mfma_signs(w.x, b0, acc0, c22, scale_b);
                acc1 = mfma_signs(w.y, b0, acc1, c22, scale_b);
                acc0 = mfma_signs(w.z, b1, acc0, c22, scale_b);
                acc1 = mfma_signs(w.w, b1, acc1, c22, scale_b);
                if (++c_tile == n_tiles) {
                    // the unit's partial sums: one entry per (row tile, chunk)
                    v4f v;
#pragma unroll
                    for (int r = 0; r < 4; ++r) v[r] = quad_sum((quad & 1) ? acc1[r] : acc0[r]);
                    if (part_writer)
                        asm volatile("ds_write_b128 %0, %1\n\ts_waitcnt lgkmcnt(0)"
                                     :
                                     : "v"(part_lane + ((cu.w2 >> UNIT_PART_SHIFT) & 0xfffu) * (uint32_t)Lds::PART_ENTRY), "v"(v)
                                     : "memory");
                    acc0 = (v4f){0, 0, 0, 0};
                    acc1 = (v4f){0, 0, 0, 0};
                    // through with the phase: its partial sums are in LDS, its tiles read
                    if ((cu.w2 & UNIT_LAST) && lane == 0) ctrl_add(ctrl + 4 * (CTRL_DONE + p % NPAR), 1u);
                    c_tile = 0u;
                    ++ci;
                    if (ci - blk0 == 64u) next_block();      // on to the next 64 records
                    cu = unit_at(ci);
                }
                issue(B[s], soff[s], stale[s]);
            }
        }
    } else {
        // ========================= finishing wavefront ======================
        const int f = wave - NL - NC;
        // lane -> (slot, sub, row): a wavefront finishes two slots per phase, one per half of its
        // lanes.  Two tokens: sub is the lane's token.  One token: the two lanes of a row split the
        // paths between them (sub = which path) for the sums and the expansion.
        const int half = lane >> 5;
        const int my_slot = 2 * f + half;
        const int row = lane & 15, sub = (lane >> 4) & 1;
        constexpr bool SPLIT = TT == 1;
        constexpr int ENTRY = Lds::PART_ENTRY / 4;              // floats per partial sum entry: [path][token][row]
        typedef __attribute__((address_space(1))) const _Float16 *gptr_h;
        uint8_t *stage = lds + Lds::STAGE_OFF + f * Lds::STAGE_WAVE;
        const float *part = reinterpret_cast<const float *>(lds + Lds::PART_OFF);
        uint32_t consumed = 0;
        uint32_t limit = SPIN_LIMIT;                          // polls a wait may take; 1 once a wait has run out
        uint32_t want0 = 0, want1 = 0;                        // consuming wavefronts expected per parity, running totals
        static_assert(NPAR == 2, "one running total per parity");
        const float pick1 = sub ? 1.f : 0.f, pick0 = 1.f - pick1;

        // Nothing on the way from the partial sums to the stores waits for memory.  The scales of
        // this lane's row come straight from HBM (a couple of microseconds), so they are requested
        // two phases ahead and only looked at when their phase is finished; the plan's scalars that
        // say where they are (PlanV) are requested a phase before that, and those the epilogue
        // itself needs (PlanE) one phase ahead.
        struct PlanV { int rt0, nrt, out, n_cons; uint64_t g, h[MAX_CONS]; };
        struct PlanE {
            int rt0, nrt, out, n_cons, nch, tiles;
            float inv_sc0, inv_sc1, sc0[MAX_CONS], sc1[MAX_CONS];
            uint64_t y, up[MAX_CONS];
        };
        struct Raw { _Float16 g0, g1, h0[MAX_CONS], h1[MAX_CONS]; };      // one token: g0 / h0 hold this lane's path
        auto fetch_v = [&](int q) -> PlanV {
            q = min(q, n_phases - 1);
            const Phase *ph = phases + q;
            const Share sh = shares[(size_t)q * G + grp];
            PlanV V;
            V.rt0 = sh.rt0; V.nrt = sh.nrt; V.out = ph->out; V.n_cons = ph->n_cons; V.g = ph->g;
#pragma unroll
            for (int c = 0; c < MAX_CONS; ++c) V.h[c] = ph->cons[c].h;
            return V;
        };
        auto fetch_e = [&](int q) -> PlanE {
            q = min(q, n_phases - 1);
            const Phase *ph = phases + q;
            const Share sh = shares[(size_t)q * G + grp];
            PlanE E;
            E.rt0 = sh.rt0; E.nrt = sh.nrt; E.out = ph->out; E.n_cons = ph->n_cons; E.nch = ph->n_chunks;
            E.tiles = sh.nrt * ph->CT;
            E.inv_sc0 = ph->inv_sc[0]; E.inv_sc1 = ph->inv_sc[1];
            E.y = ph->y;
#pragma unroll
            for (int c = 0; c < MAX_CONS; ++c) {
                E.up[c] = ph->cons[c].up;
                E.sc0[c] = ph->cons[c].sc[0]; E.sc1[c] = ph->cons[c].sc[1];
            }
            return E;
        };
        auto load_raw = [&](const PlanV &V) -> Raw {      // loads only: nothing here may look at what it loaded
            Raw R;
            R.g0 = 0; R.g1 = 0;
#pragma unroll
            for (int c = 0; c < MAX_CONS; ++c) { R.h0[c] = 0; R.h1[c] = 0; }
            if (my_slot < V.nrt) {
                const gptr_h g = (gptr_h)V.g;
                const int gi = min((V.rt0 + my_slot) * 16 + row, V.out - 1);      // a reader's width is the op's height
                if constexpr (SPLIT) {
                    R.g0 = g[(size_t)sub * V.out + gi];
                } else {
                    R.g0 = g[gi];
                    R.g1 = g[(size_t)V.out + gi];
                }
#pragma unroll
                for (int c = 0; c < MAX_CONS; ++c) {
                    if (c < V.n_cons) {
                        const gptr_h h = (gptr_h)V.h[c];
                        if constexpr (SPLIT) {
                            R.h0[c] = h[(size_t)sub * V.out + gi];
                        } else {
                            R.h0[c] = h[gi];
                            R.h1[c] = h[(size_t)V.out + gi];
                        }
                    }
                }
            }
            return R;
        };

        // one phase: wait for its partial sums, finish this wavefront's rows
        auto finish = [&](int q, const PlanE &E, const Raw &R) {
            const int nrt = E.nrt, out = E.out, n_cons = E.n_cons, nch = E.nch;
            const bool have = my_slot < nrt;
            const int grow = (E.rt0 + my_slot) * 16 + row;
            const bool active = have && grow < out;
            // ---- wait until every consuming wavefront that has a unit in the phase is through with
            // it: units are dealt c * U / NC, so min(U, NC) wavefronts have one (running total per parity)
            {
                const uint32_t with_units = (uint32_t)min(nrt * nch, NC);
                uint32_t want;
                if (q % NPAR == 0) want = (want0 += with_units);
                else want = (want1 += with_units);
                if (with_units != 0u && wait_word(ctrl + 4 * (CTRL_DONE + q % NPAR), want, limit) < want) {
                    limit = 1;
                    give_up();
                }
            }
            consumed += (uint32_t)E.tiles;
            if (f == 0 && lane == 0) ctrl_write(ctrl + 4 * CTRL_CONSUMED, consumed);      // the phase's ring slots are free

            // a_k = g_k / sc_k of the op, hs = h_k * sc_k of each reader (one token: this lane's path only)
            float a0, a1 = 0.f, hs0[MAX_CONS], hs1[MAX_CONS];
            if constexpr (SPLIT) {
                // this lane's path: picked with weights 0 and 1 (exact: the scales are finite powers of
                // two), because a lane-dependent choice between two members of the plan would be
                // compiled into an array in scratch memory indexed by the lane
                a0 = (float)R.g0 * (pick0 * E.inv_sc0 + pick1 * E.inv_sc1);
#pragma unroll
                for (int c = 0; c < MAX_CONS; ++c) { hs0[c] = (float)R.h0[c] * (pick0 * E.sc0[c] + pick1 * E.sc1[c]); hs1[c] = 0.f; }
            } else {
                a0 = (float)R.g0 * E.inv_sc0;
                a1 = (float)R.g1 * E.inv_sc1;
#pragma unroll
                for (int c = 0; c < MAX_CONS; ++c) { hs0[c] = (float)R.h0[c] * E.sc0[c]; hs1[c] = (float)R.h1[c] * E.sc1[c]; }
            }

            // ---- a3/a4: partial sums of the row in chunk order, output scales, path sum, one rounding
            float yf = 0.f;
            if (have) {
                const float *PS = part + (size_t)(((q % NPAR) * MAX_SLOTS + my_slot) * MAX_CHUNKS) * ENTRY + row;
                if constexpr (SPLIT) {
                    float mine = 0.f;
                    for (int ch = 0; ch < nch; ++ch) mine += PS[ch * ENTRY + sub * 16];
                    const float other = __shfl_xor(mine, 16);        // the lane with the same row and the other path
                    const float a_other = __shfl_xor(a0, 16);
                    const float s0 = sub ? other : mine, s1 = sub ? mine : other;
                    const float g0 = sub ? a_other : a0, g1 = sub ? a0 : a_other;
                    const _Float16 y16 = (_Float16)path_sum(g0, s0, g1, s1);      // round to nearest even
                    if (active && sub == 0) ((__attribute__((address_space(1))) _Float16 *)E.y)[grow] = y16;
                    yf = (float)y16;
                } else {
                    float s0 = 0.f, s1 = 0.f;
                    for (int ch = 0; ch < nch; ++ch) {
                        s0 += PS[ch * ENTRY + (0 * TT + sub) * 16];
                        s1 += PS[ch * ENTRY + (1 * TT + sub) * 16];
                    }
                    const _Float16 y16 = (_Float16)path_sum(a0, s0, a1, s1);
                    if (active) ((__attribute__((address_space(1))) _Float16 *)E.y)[(size_t)sub * out + grow] = y16;
                    yf = (float)y16;
                }
            }
            // ---- a1 for the readers: h (.) y as four bf8 terms; the bytes of 16 rows make one 16-byte
            // group.  Rows beyond the end of the matrix stage zero bytes (padding columns of the reader).
            if (n_cons > 0) {
                if (have) {
#pragma unroll
                    for (int c = 0; c < MAX_CONS; ++c) {
                        if (c < n_cons) {
                            if constexpr (SPLIT) {
                                const uint32_t terms = active ? expand4(hs0[c] * yf) : 0u;
                                uint8_t *dst = stage + (((half * MAX_CONS + c) * 2 + sub) * 4) * 16 + row;      // [half][reader][path][term][row]
#pragma unroll
                                for (int t = 0; t < 4; ++t) dst[t * 16] = (uint8_t)(terms >> (8 * t));
                            } else {
#pragma unroll
                                for (int p = 0; p < 2; ++p) {
                                    const uint32_t terms = active ? expand4((p ? hs1[c] : hs0[c]) * yf) : 0u;
                                    uint8_t *dst = stage + ((((half * MAX_CONS + c) * TT + sub) * 2 + p) * 4) * 16 + row;   // [half][reader][token][path][term][row]
#pragma unroll
                                    for (int t = 0; t < 4; ++t) dst[t * 16] = (uint8_t)(terms >> (8 * t));
                                }
                            }
                        }
                    }
                }
                // lanes now act as (half, reader, operand column = 8 token + 4 path + term): vectors of 16 bytes
                constexpr int COLS = TT * 8, VECS = 2 * MAX_CONS * COLS;
#pragma unroll
                for (int round = 0; round < (VECS + 63) / 64; ++round) {
                    const int v = lane + 64 * round;
                    const int vh = v / (MAX_CONS * COLS), vc = (v / COLS) % MAX_CONS, vcol = v % COLS;
                    const int slot_v = 2 * f + vh;
                    if (v < VECS && slot_v < nrt && vc < n_cons) {
                        // (masks, not a choice between members of the plan: see the note on pick0 / pick1)
                        const uint64_t m1 = 0ull - (uint64_t)(vc == 1), m2 = 0ull - (uint64_t)(vc == 2);
                        const uint64_t base = (E.up[0] & ~(m1 | m2)) | (E.up[1] & m1) | (E.up[2] & m2);
                        const v4i bytes = *reinterpret_cast<const v4i *>(stage + (size_t)v * 16);
                        uint8_t *dst = reinterpret_cast<uint8_t *>(base) + up_group_offset(TT, (E.rt0 + slot_v) * 16, 0) + (size_t)vcol * 16;
                        asm volatile("global_store_dwordx4 %0, %1, off sc1" : : "v"(dst), "v"(bytes) : "memory");
                    }
                }
            }
            // ---- this phase's outputs are on their way
            if (lane == 0) {
                if (f == 0) ctrl_write(ctrl + 4 * (CTRL_FIN_TIME + (q & 7)), clock32());
                ctrl_write(ctrl + 4 * (CTRL_FIN + f), (uint32_t)q + 1u);
            }
        };

        // three sets of row scales rotate through the loop (its body covers three phases, so that
        // no set is ever copied: a copy would wait for the loads that fill it)
        PlanE e_cur = fetch_e(0);
        Raw r0 = load_raw(fetch_v(0)), r1 = load_raw(fetch_v(1)), r2 = r0;
        PlanV v_ahead = fetch_v(2);
        for (int q = 0; q < n_phases; q += 3) {
            {
                const PlanE e_nxt = fetch_e(q + 1);
                const PlanV v_nxt = fetch_v(q + 3);
                r2 = load_raw(v_ahead);
                finish(q, e_cur, r0);
                e_cur = e_nxt;
                v_ahead = v_nxt;
            }
            if (q + 1 < n_phases) {
                const PlanE e_nxt = fetch_e(q + 2);
                const PlanV v_nxt = fetch_v(q + 4);
                r0 = load_raw(v_ahead);
                finish(q + 1, e_cur, r1);
                e_cur = e_nxt;
                v_ahead = v_nxt;
            }
            if (q + 2 < n_phases) {
                const PlanE e_nxt = fetch_e(q + 3);
                const PlanV v_nxt = fetch_v(q + 5);
                r1 = load_raw(v_ahead);
                finish(q + 2, e_cur, r2);
                e_cur = e_nxt;
                v_ahead = v_nxt;
            }
        }
        // after the last phase nobody waits for a tile any more
        if (f == 0 && lane == 0) {
            const uint32_t again = ctrl_read(ctrl + 4 * CTRL_WAITED);
            if (again != 0)
                __hip_atomic_fetch_add(RB_GLOBAL(uint32_t, error) + 1, again, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// ------------------------------------------------------------------ host ---
static Layout make_layout(int n_ops, int n_phases, int n_groups, size_t unit_stride, size_t up_total)
{
    Layout L;
    size_t o = sizeof(Header);
    o = align_up(o, 128); L.ops = o; o += sizeof(Op) * (size_t)n_ops;
    o = align_up(o, 128); L.seeds = o; o += sizeof(PhaseSeed) * (size_t)n_phases;
    o = align_up(o, 128); L.error = o; o += 128;
    L.which = o; o += align_up(sizeof(int) * MAX_EXPAND, 128);
    o = align_up(o, 256); L.phases = o; o += sizeof(Phase) * (size_t)n_phases;
    o = align_up(o, 256); L.shares = o; o += sizeof(Share) * (size_t)n_phases * (size_t)n_groups;
    o = align_up(o, 256); L.units = o; o += sizeof(Unit) * unit_stride * (size_t)NC * (size_t)n_groups;
    o = align_up(o, 256); L.up = o; o += up_total;
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
    // a row tile's share of one workgroup must fit the ring of sign tiles
    return L->K == 2 && T >= 1 && T <= MAX_T && L->in % 32 == 0 && col_tiles(L->in) <= RING_TILES &&
           chunk_tiles(col_tiles(L->in)) <= 255;
}

// row tiles of one op that a phase may hold: a workgroup's share is at most MAX_SLOTS row tiles and
// at most RING_TILES sign tiles
static int phase_row_tiles(int RT, int CT, int G)
{
    const int per_group = std::max(1, std::min(MAX_SLOTS, RING_TILES / CT));
    const int pieces = (RT + per_group * G - 1) / (per_group * G);
    return (RT + pieces - 1) / pieces;
}
static int phases_of(int RT, int CT, int G)
{
    const int n = phase_row_tiles(RT, CT, G);
    return (RT + n - 1) / n;
}
// units one consuming wavefront can have in one phase of n_rt row tiles: its part of the largest share
static int wave_units(int n_rt, int CT, int G)
{
    const int share = (n_rt + G - 1) / G;
    return (share * chunks_of(CT) + NC - 1) / NC;
}

size_t plan_workspace_bytes(const rb_layer *layers, int n_layers, int n_ops, int T)
{
    // upper bound: every op could use the widest layer and the layer that needs the most phases
    size_t up_max = 0;
    int G = device_groups();
    if (G <= 0) G = 256;       // no device to ask (size queries on a host): an MI355X
    int phases_max = 1, units_max = 1;
    for (int l = 0; l < n_layers; ++l) {
        const int RT = row_tiles(layers[l].out), CT = col_tiles(layers[l].in);
        up_max = std::max(up_max, up_bytes(layers[l].in, T));
        phases_max = std::max(phases_max, phases_of(RT, CT, G));
        units_max = std::max(units_max, phases_of(RT, CT, G) * wave_units(phase_row_tiles(RT, CT, G), CT, G));
    }
    // size queries made without a device must not come out smaller than with one: bound the groups from above
    const int G_bound = std::max(G, 1024);
    return make_layout(n_ops, n_ops * phases_max, G_bound, align_up((size_t)n_ops * units_max + 1, 64) + 64,
                       align_up(up_max, 256) * (size_t)n_ops)
        .total;
}

// Host record of a prepared plan, keyed by the workspace that holds its device part.
struct Prepared {
    Layout lay;
    int n_ops = 0, n_phases = 0, G = 0, T = 0, max_expand_in = 0, n_expand = 0, unit_stride = 0;
    size_t up_total = 0;
    bool dependent = false;                 // some op reads what another op of the launch writes
    int pause_clks = 0;
    std::vector<uint8_t> blob;              // what prepare uploads; kept while its copy may be pending
    std::vector<int> which;
};
static std::mutex g_mutex;
static std::map<const void *, Prepared> g_prepared;
static int g_pause_clks = 1400;             // see rb_stack_set_pause

void set_pause(int clks)
{
    std::lock_guard<std::mutex> lock(g_mutex);
    g_pause_clks = std::max(0, std::min(clks, 1 << 20));
}

// Order of the ops: list scheduling on the dependency graph.  An op may start once its producer
// has been placed; its input is taken to arrive `latency` after the producer's last phase (in
// units of sign tiles per workgroup, the measure of an op's duration).  At every step the op
// with the longest chain of dependent work behind it goes first among those whose input has
// arrived; when none has, the op that becomes ready first.  Ops nobody waits for thus land in the
// gaps that hand-overs leave.
static std::vector<int> schedule_ops(const std::vector<Op> &ops, int G)
{
    const int n = (int)ops.size();
    constexpr double LATENCY = 40.0;
    std::vector<double> dur((size_t)n), tail((size_t)n, 0.0);
    for (int i = 0; i < n; ++i) dur[(size_t)i] = (double)ops[(size_t)i].RT * ops[(size_t)i].CT / G;
    for (int i = n - 1; i >= 0; --i) {                        // consumers have larger indices
        double t = 0.0;
        for (int c = 0; c < ops[(size_t)i].n_cons; ++c) t = std::max(t, LATENCY + tail[(size_t)ops[(size_t)i].cons[c]]);
        tail[(size_t)i] = dur[(size_t)i] + t;
    }
    std::vector<int> order;
    std::vector<char> placed((size_t)n, 0);
    std::vector<double> finish((size_t)n, 0.0);
    double now = 0.0;
    // the candidates are searched in a window behind the first unplaced op: a plan keeps the
    // caller's order except where an op can fill a gap
    int first = 0;
    constexpr int WINDOW = 64;
    while ((int)order.size() < n) {
        while (first < n && placed[(size_t)first]) ++first;
        int best = -1, soonest = -1;
        double soonest_t = 0.0;
        for (int i = first; i < n && i < first + WINDOW; ++i) {
            if (placed[(size_t)i]) continue;
            const int d = ops[(size_t)i].dep;
            if (d >= 0 && !placed[(size_t)d]) continue;
            const double ready = d >= 0 ? finish[(size_t)d] + LATENCY : 0.0;
            if (ready <= now) {
                if (best < 0 || tail[(size_t)i] > tail[(size_t)best]) best = i;
            } else if (soonest < 0 || ready < soonest_t) {
                soonest = i;
                soonest_t = ready;
            }
        }
        const int pick = best >= 0 ? best : soonest;
        if (best < 0) now = soonest_t;
        placed[(size_t)pick] = 1;
        now += dur[(size_t)pick];
        finish[(size_t)pick] = now;
        order.push_back(pick);
    }
    return order;
}

int prepare_plan(const rb_layer *layers, const rb_stack_op *sops, int n_ops, uint16_t *const *bufs, int T,
                 void *workspace, size_t workspace_bytes_, hipStream_t stream)
{
    const int G = device_groups();
    if (G <= 0) return RB_ERR_HIP;
    if (n_ops > MAX_OPS) return RB_ERR_UNSUPPORTED;

    // ---- ops and who reads whose output
    std::vector<Op> ops((size_t)n_ops);
    std::vector<int> expand_list;
    size_t up_total = 0;
    std::vector<size_t> up_off((size_t)n_ops);
    bool dependent = false;
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
        o.dep = producer;
        if (producer < 0) {
            o.expand_x = 1;
            expand_list.push_back(n);
        } else {
            Op &pr = ops[(size_t)producer];
            if (pr.n_cons >= MAX_CONS) return RB_ERR_UNSUPPORTED;
            if (pr.out != o.in) return RB_ERR_SHAPE;
            pr.cons[pr.n_cons++] = n;
            dependent = true;
        }
        // Reordering is safe for what ops read: every op has an expanded input of its own, written
        // by its producer only (or before the launch, from the buffer as the caller left it).  Two
        // ops that write the same buffer keep their meaning only in the caller's order: such lists
        // are left to the general path.
        for (int m = 0; m < n; ++m)
            if (sops[m].dst == sops[n].dst) return RB_ERR_UNSUPPORTED;
    }
    if (expand_list.size() > MAX_EXPAND) return RB_ERR_UNSUPPORTED;

    // ---- phases, in the planner's order
    const std::vector<int> order = schedule_ops(ops, G);
    std::vector<PhaseSeed> seeds;
    for (int n : order) {
        Op &o = ops[(size_t)n];
        const int per_phase = phase_row_tiles(o.RT, o.CT, G);
        for (int rt = 0; rt < o.RT; rt += per_phase) {
            PhaseSeed sd;
            sd.op = n;
            sd.rt_first = rt;
            sd.n_rt = std::min(per_phase, o.RT - rt);
            // the larger shares of a phase (when G does not divide its row tiles) start at a
            // different workgroup from phase to phase
            sd.rot = (int)((seeds.size() * 37u) % (unsigned)G);
            seeds.push_back(sd);
        }
        o.last_phase = (int)seeds.size() - 1;
    }
    const int n_phases = (int)seeds.size();
    if (n_phases > MAX_PHASES || up_total >= ((size_t)1 << 31)) return RB_ERR_UNSUPPORTED;
    // records per wavefront: its units, an end mark, and padding so that the list can be read 64
    // records at a time, one block ahead
    size_t unit_stride = 1;
    for (const PhaseSeed &sd : seeds) unit_stride += (size_t)wave_units(sd.n_rt, ops[(size_t)sd.op].CT, G);
    unit_stride = align_up(unit_stride, 64) + 64;

    Prepared pr;
    pr.n_ops = n_ops; pr.n_phases = n_phases; pr.G = G; pr.T = T;
    pr.n_expand = (int)expand_list.size();
    pr.dependent = dependent;
    for (int n : expand_list) pr.max_expand_in = std::max(pr.max_expand_in, ops[(size_t)n].in);
    pr.unit_stride = (int)unit_stride;
    pr.up_total = up_total;
    pr.lay = make_layout(n_ops, n_phases, G, unit_stride, up_total);
    const Layout &lay = pr.lay;
    if (workspace_bytes_ < lay.total) return RB_ERR_WORKSPACE;
    uint8_t *ws = static_cast<uint8_t *>(workspace);
    for (int n = 0; n < n_ops; ++n) ops[(size_t)n].up = ws + lay.up + up_off[(size_t)n];

    Header hdr{};
    hdr.n_ops = n_ops; hdr.n_phases = n_phases; hdr.T = T; hdr.n_groups = G;
    hdr.unit_stride = (int)unit_stride;

    // ---- upload: stream-ordered copies out of host memory that lives as long as the plan's record
    pr.blob.assign(lay.error, 0);
    std::memcpy(pr.blob.data(), &hdr, sizeof(hdr));
    std::memcpy(pr.blob.data() + lay.ops, ops.data(), sizeof(Op) * (size_t)n_ops);
    std::memcpy(pr.blob.data() + lay.seeds, seeds.data(), sizeof(PhaseSeed) * (size_t)n_phases);
    pr.which = expand_list;
    Prepared *rec;
    {
        std::lock_guard<std::mutex> lock(g_mutex);
        pr.pause_clks = g_pause_clks;
        rec = &(g_prepared[workspace] = std::move(pr));
    }
    if (hipMemcpyAsync(ws, rec->blob.data(), lay.error, hipMemcpyHostToDevice, stream) != hipSuccess) return RB_ERR_HIP;
    if (!rec->which.empty() &&
        hipMemcpyAsync(ws + lay.which, rec->which.data(), sizeof(int) * rec->which.size(), hipMemcpyHostToDevice, stream) !=
            hipSuccess)
        return RB_ERR_HIP;
    hipLaunchKernelGGL(prep_kernel, dim3(n_ops), dim3(256), 0, stream, reinterpret_cast<const Header *>(ws),
                       reinterpret_cast<Op *>(ws + lay.ops), reinterpret_cast<uint32_t *>(ws + lay.error));
    hipLaunchKernelGGL(phase_kernel, dim3(n_phases), dim3(256), 0, stream, reinterpret_cast<const Header *>(ws),
                       reinterpret_cast<const Op *>(ws + lay.ops), reinterpret_cast<const PhaseSeed *>(ws + lay.seeds),
                       reinterpret_cast<Phase *>(ws + lay.phases), reinterpret_cast<Share *>(ws + lay.shares));
    hipLaunchKernelGGL(unit_kernel, dim3((G * NC + 63) / 64), dim3(64), 0, stream, reinterpret_cast<const Header *>(ws),
                       reinterpret_cast<const Phase *>(ws + lay.phases), reinterpret_cast<const Share *>(ws + lay.shares),
                       ws + lay.up, reinterpret_cast<Unit *>(ws + lay.units));
    return hipGetLastError() == hipSuccess ? RB_OK : RB_ERR_HIP;
}

int launch_plan(void *workspace, size_t workspace_bytes_, hipStream_t stream)
{
    int n_ops, n_phases, G, T, n_expand, max_expand_in, pause, unit_stride;
    size_t up_total;
    bool dependent;
    Layout lay;
    {
        std::lock_guard<std::mutex> lock(g_mutex);
        const auto it = g_prepared.find(workspace);
        if (it == g_prepared.end()) return RB_ERR_WORKSPACE;
        const Prepared &pr = it->second;
        n_ops = pr.n_ops; n_phases = pr.n_phases; G = pr.G; T = pr.T; n_expand = pr.n_expand;
        max_expand_in = pr.max_expand_in; dependent = pr.dependent; lay = pr.lay; pause = pr.pause_clks;
        unit_stride = pr.unit_stride; up_total = pr.up_total;
    }
    if (workspace_bytes_ < lay.total) return RB_ERR_WORKSPACE;
    uint8_t *ws = static_cast<uint8_t *>(workspace);
    const Header *d_hdr = reinterpret_cast<const Header *>(ws);
    const Op *d_ops = reinterpret_cast<const Op *>(ws + lay.ops);
    if (n_expand > 0)
        hipLaunchKernelGGL(expand_kernel, dim3((max_expand_in + 255) / 256, T, (unsigned)n_expand), dim3(256), 0, stream,
                           d_hdr, d_ops, reinterpret_cast<const int *>(ws + lay.which));
    if (dependent) hipLaunchKernelGGL(poison_kernel, dim3(n_ops, POISON_SPLIT), dim3(256), 0, stream, d_ops, T);
    auto launch = [&](auto kernel, int lds_bytes) -> int {
        // once per device and kernel: allow the LDS request
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                lds_bytes) != hipSuccess)
            return RB_ERR_HIP;
        hipLaunchKernelGGL(kernel, dim3(G), dim3(THREADS), lds_bytes, stream,
                           reinterpret_cast<const Phase *>(ws + lay.phases), reinterpret_cast<const Share *>(ws + lay.shares),
                           reinterpret_cast<const Unit *>(ws + lay.units), unit_stride, ws + lay.up, (uint32_t)up_total,
                           n_phases, reinterpret_cast<uint32_t *>(ws + lay.error), pause);
        return RB_OK;
    };
    const int rc = T == 1 ? launch(chain_kernel<1>, LdsMap<1>::BYTES) : launch(chain_kernel<2>, LdsMap<2>::BYTES);
    if (rc != RB_OK) return rc;
    return hipGetLastError() == hipSuccess ? RB_OK : RB_ERR_HIP;
}

int plan_status(const void *workspace, hipStream_t stream, unsigned long long *waited)
{
    size_t error_off;
    {
        std::lock_guard<std::mutex> lock(g_mutex);
        const auto it = g_prepared.find(workspace);
        if (it == g_prepared.end()) return RB_ERR_WORKSPACE;
        error_off = it->second.lay.error;
    }
    uint32_t mark[2] = {0, 0};               // gave up a wait; tiles read again
    if (hipMemcpyAsync(mark, static_cast<const uint8_t *>(workspace) + error_off, sizeof(mark), hipMemcpyDeviceToHost,
                       stream) != hipSuccess ||
        hipStreamSynchronize(stream) != hipSuccess)
        return RB_ERR_HIP;
    if (waited) *waited += mark[1];
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
