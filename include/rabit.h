/*
 * rabit.h - C ABI of the residual-binary linear layer for AMD MI355X (gfx950).
 *
 * The layer (paper Section 4.1 "Binary Building Blocks" and Eq. "stacked binary
 * weight"):
 *
 *      y = sum_{k=1..K}  g_k (.) ( B_k ( h_k (.) x ) )
 *
 * B_k in {-1,+1}^{out x in} is stored as sign bits, g_k (length out) scales the
 * output channels and h_k (length in) the input channels of path k.  (The code
 * listing in the paper's last appendix names the two scale vectors the other
 * way round; this library follows Section 4.1.)
 *
 * Conventions for every function
 *   - returns RB_OK (0) or a negative RB_ERR_* code; never throws or aborts;
 *   - "host" pointers are ordinary CPU memory, "device" pointers are HIP device
 *     memory of the current device; the caller owns every buffer;
 *   - compute functions only enqueue work on `stream` (a hipStream_t passed as
 *     void*, NULL = the default stream); they do not synchronise and do not
 *     allocate.  Scratch memory comes from the caller as `workspace`;
 *   - activations and scales are IEEE binary16 bit patterns (uint16_t) unless a
 *     dtype argument says otherwise; accumulation is fp32;
 *   - token-major layout for batches: X[T][in], Y[T][out] (the layout of the
 *     paper's host wrapper: x is [seqlen, in], y is [seqlen, out]).
 */
#ifndef RABIT_H
#define RABIT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define RB_OK               0
#define RB_ERR_NULL        -1   /* a required pointer is NULL                         */
#define RB_ERR_SHAPE       -2   /* in % 32 != 0, K outside 1..RB_MAX_K, T < 1, ...    */
#define RB_ERR_ALIGN       -3   /* a device pointer is not 16-byte aligned            */
#define RB_ERR_UNSUPPORTED -4   /* valid request this build has no kernel for         */
#define RB_ERR_HIP         -5   /* the HIP runtime reported an error on launch        */
#define RB_ERR_WORKSPACE   -6   /* workspace missing or smaller than rb_workspace_bytes */
#define RB_ERR_VALUE       -7   /* rb_pack: an entry is neither +1 nor -1             */
#define RB_ERR_HANDOVER    -8   /* rb_stack_status: a run gave up waiting for another compute unit */

/* K = 2 is the 2-bit layer every kernel here is built for.  K = 3 (the 3-bit variant of the
 * paper's packing appendix): stacks run on the matrix cores (one token on the fused decode kernel,
 * 2..16 tokens on the small-batch kernel), single calls of 6 tokens or more too (the small-batch
 * kernel up to 12 fp16 tokens, the many-token kernel otherwise), shorter single calls on the
 * generic sign-XOR + add kernel, which also runs K = 1. */
#define RB_MAX_K 3

/* element types for rb_linear_gemm */
#define RB_F16  0
#define RB_BF16 1
#define RB_F32  2

/* ------------------------------------------------------------------------
 * Packing (host, pure CPU, bit-exact).  Appendix "Weight Packing": every group
 * of 32 columns becomes one 32-bit word, +1 -> bit 0, -1 -> bit 1.  Canonical
 * form: word w of row i of path k holds columns 32w..32w+31, least-significant
 * bit = lowest column; array uint32 [K][out][in/32], row-major.
 * signs: int8 [K][out][in], entries +1 or -1.  Requires in % 32 == 0.
 * ------------------------------------------------------------------------ */
int rb_pack(const int8_t *signs, int K, int out, int in, uint32_t *packed);
int rb_unpack(const uint32_t *packed, int K, int out, int in, int8_t *signs);

/*
 * Kernel-native layout (the same appendix interleaves rows so that a wavefront
 * issues full coalesced loads; this is that idea laid out for 64-lane
 * wavefronts and 128-bit loads).  The matrix is cut into tiles of 16 rows by
 * 256 columns; rows are padded to a multiple of 16 and columns to a multiple
 * of 256 with +1 entries (bit 0).  Tiles are stored row-tile major.  Inside a
 * tile, lane l = r + 16*q (r = row in tile, q = 0..3) owns 2*K consecutive
 * words: for c in {0,1}, for k in 0..K-1: the word of path k, row r, columns
 * 128*c + 32*q .. +31 of the tile, with its 32 columns bit-interleaved: native
 * bit 4*e + s (e = 0..7, s = 0..3) is column 8*s + e.  One tile is 64 * 2K words.
 * rb_native_bytes gives the size; rb_repack_native / rb_unpack_native convert
 * host arrays between the canonical and the native form (exact inverses on the
 * unpadded part).
 */
size_t rb_native_bytes(int K, int out, int in);
int rb_repack_native(const uint32_t *packed, int K, int out, int in, void *native_host);
int rb_unpack_native(const void *native_host, int K, int out, int in, uint32_t *packed);

/* One frozen layer as the kernels consume it (Section 4.2, last paragraph: the
 * binary cores are frozen for inference and the full-precision weight is gone). */
typedef struct rb_layer {
    int out, in, K;
    const void     *bits;   /* device, native layout, rb_native_bytes(K,out,in) bytes, 16B aligned */
    const uint16_t *g;      /* device fp16 [K][out] */
    const uint16_t *h;      /* device fp16 [K][in]  */
} rb_layer;

/*
 * Decode GEMV, one token:  y = sum_k g_k (.) (B_k (h_k (.) x)).
 * x device fp16 [in], y device fp16 [out] (round-to-nearest-even from fp32).
 * Equals rb_linear_gemm with T = 1, RB_F16 in and out.
 */
int rb_linear_gemv(const rb_layer *L, const uint16_t *x, uint16_t *y,
                   void *workspace, size_t workspace_bytes, void *stream);

/*
 * Batched form, T tokens: Y[t] = layer(X[t]).  X device [T][in] of act_dtype
 * (RB_F16 or RB_BF16), Y device [T][out] of out_dtype (RB_F16, RB_BF16, RB_F32).
 * Small T streams the weights once for all tokens; large T runs as a dense
 * contraction on the matrix cores: beyond 32 tokens as Y = W_hat X with the
 * effective weight W_hat = sum_k g_k (.) B_k (.) h_k (the form Alg. 2 gives for
 * batched inputs), which the kernel builds in fp16 registers from the packed
 * signs (two roundings per weight, a few 1e-4 relative on the output; fp32
 * accumulation).
 */
int rb_linear_gemm(const rb_layer *L, const void *X, void *Y, int T,
                   int act_dtype, int out_dtype,
                   void *workspace, size_t workspace_bytes, void *stream);

/*
 * rb_linear_gemm for callers that cannot allocate or hold a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and
 * status codes as rb_linear_gemm without the workspace pair; the scratch memory of the many-token
 * kernel is a device array inside the library (RB_NOALLOC_SCRATCH_BYTES per GPU that uses the
 * library, held until the process ends).  The call allocates nothing on host or device.  It returns
 * RB_ERR_WORKSPACE when rb_workspace_bytes(L, 1, 1, T) of the many-token kernel exceeds
 * RB_NOALLOC_SCRATCH_BYTES (roughly T_padded * in above 4 M elements; a three-path layer at up to
 * 32 tokens takes the generic kernel then, which needs no scratch memory, and where the variant
 * with a workspace takes the small-batch kernel this one takes the many-token kernel: same result
 * to the tolerance, not bit for bit).  Every call on one GPU
 * shares that GPU's array: calls that may overlap in time on one GPU (different streams or
 * threads) race and must be ordered by the caller; calls on one stream are ordered already.
 * rb_noalloc_scratch_bytes returns RB_NOALLOC_SCRATCH_BYTES.
 */
#define RB_NOALLOC_SCRATCH_BYTES (32u << 20)
int rb_linear_gemm_noalloc(const rb_layer *L, const void *X, void *Y, int T,
                           int act_dtype, int out_dtype, void *stream);
size_t rb_noalloc_scratch_bytes(void);

/*
 * A stack of layers run in order (the end-to-end decode setting of the paper's
 * inference table, reduced to its linear layers).  Op n applies
 * layers[ops[n].layer] to bufs[ops[n].src] and writes bufs[ops[n].dst]; every
 * buffer is device fp16 [T][width].  The result of each op equals
 * rb_linear_gemm on the same input (bit for bit for T <= 2 and T > 16; for
 * 3 <= T <= 16 a stack runs on the fused decode kernel or the small-batch
 * kernel while a single call takes the many-token kernel, and they agree to the
 * accuracy all are held to).  An op may read any buffer written by an
 * earlier op (or never written: stack inputs); dst buffers must be distinct
 * from the op's src.  layers, ops and bufs are host arrays; bufs holds n_bufs
 * device pointers.  Activations are expected to be finite: an infinity or NaN
 * in an op's input (an fp16 overflow upstream) makes that op's outputs NaN on
 * the fused kernels, where plain arithmetic could still give an infinity.
 */
typedef struct rb_stack_op { int layer; int src; int dst; } rb_stack_op;

int rb_layer_stack(const rb_layer *layers, int n_layers,
                   const rb_stack_op *ops, int n_ops,
                   uint16_t *const *bufs, int n_bufs, int T,
                   void *workspace, size_t workspace_bytes, void *stream);

/*
 * The same stack split for decode loops: rb_stack_prepare does everything that
 * depends only on the frozen layers, the op list and the buffer addresses
 * (uploads the op list into the workspace, derives per-layer constants from h,
 * clears the scratch arrays) and rb_stack_run executes the prepared ops once
 * on the current contents of the input buffers.  Between the two calls and
 * between runs the caller must not write to the workspace nor change layers,
 * buffers addresses or T; rb_stack_forget drops the library's host-side record
 * of a workspace (call it before the memory is reused for something else).
 * Two paths: T <= 4 runs as one launch; 5 <= T <= 7 as one launch per group
 * of four consecutive tokens (every layer's out a multiple of 8, at least two
 * ops); 8 <= T <= 16 on the small-batch kernel (one pass over the weights for all
 * tokens, one launch per group of independent ops).  Three paths in every
 * layer: T = 1 as one launch, 2 <= T <= 16 on the small-batch kernel, which
 * also takes stacks that mix two- and three-path layers.
 * rb_stack_prepare returns RB_ERR_UNSUPPORTED for stacks that only
 * rb_layer_stack's general path can run (K = 1, T > 16, an output read by more
 * than three ops, more than 1024 ops fed from outside the stack).
 */
int rb_stack_prepare(const rb_layer *layers, int n_layers,
                     const rb_stack_op *ops, int n_ops,
                     uint16_t *const *bufs, int n_bufs, int T,
                     void *workspace, size_t workspace_bytes, void *stream);
int rb_stack_run(void *workspace, size_t workspace_bytes, void *stream);
int rb_stack_forget(const void *workspace);
/*
 * The fused kernel hands activations from compute unit to compute unit while it
 * runs and assumes that all of its workgroups are resident at once (one per
 * compute unit of the device).  Every wait in it is bounded: if something
 * keeps a workgroup from running (compute units reserved by someone else), the
 * others stop waiting, finish with meaningless outputs and leave a mark in the
 * workspace.  rb_stack_status waits for `stream` (the only call of this library
 * that synchronises) and returns RB_ERR_HANDOVER if any run since
 * rb_stack_prepare left that mark, RB_OK otherwise, RB_ERR_WORKSPACE for a
 * workspace that holds no prepared stack.
 */
int rb_stack_status(const void *workspace, void *stream);
/*
 * Diagnostic: which bounded wait a run gave up, for a workspace whose rb_stack_status is
 * RB_ERR_HANDOVER (waits for `stream`; *reason, host: 0 none, 1 an input tile was never written,
 * 2 a tile kept reading as unwritten after its first bytes had arrived, 3 a stage was never
 * announced inside a workgroup, 4 a value of a decoder block's epilogue never arrived).
 */
int rb_stack_gave_up(const void *workspace, void *stream, int *reason);
/*
 * Diagnostic of the hand-over pacing: like rb_stack_status (waits for `stream`,
 * same return values), and stores in *tiles (host) how many input tiles, over
 * all runs since rb_stack_prepare, a wavefront found not yet written when it
 * came to use them and therefore waited for and read again.  Results do not
 * depend on it; a large count per run means time lost to such waits.
 */
int rb_stack_waited(const void *workspace, void *stream, unsigned long long *tiles);

/*
 * Tuning and test knob of the fused kernel; affects launches made afterwards (process-wide).
 * RB_OPT_HANDOVER_PAUSE: clocks (rounded down to multiples of 64) a compute unit lets pass, after
 * it has stored its own part of a group of independent ops, before it asks for the parts the other
 * compute units store.  Results never depend on it (what is read too early is detected and read
 * again); 0 makes nearly every input tile an early read, which is what the tests use it for.  A
 * negative value restores the built-in timing.  Returns RB_ERR_UNSUPPORTED for an unknown option.
 */
#define RB_OPT_HANDOVER_PAUSE 1
int rb_stack_set_option(int option, int value);

/* Bytes of workspace that a compute call over n_ops ops on these layers needs
 * at T tokens (n_ops = 1 for rb_linear_gemv / rb_linear_gemm; 16-byte aligned
 * device memory, contents owned by the library between calls). */
size_t rb_workspace_bytes(const rb_layer *layers, int n_layers, int n_ops, int T);

/* ------------------------------------------------------------------------
 * Training side (Section 4.2 "Backward Pass and Parameter Updates", Alg. 2).
 * All pointers are device pointers; nothing allocates or synchronises.
 * ------------------------------------------------------------------------ */

/*
 * On-the-fly residual coupling (Alg. 2, forward loop): from the shared weight W
 * (fp32 [out][in], 16-byte aligned) and the scales g (fp16 [K][out]), h (fp16
 * [K][in], 8-byte aligned) derive
 *   R_0 = W;  B_i = sign(R_{i-1}) (sign(0) = +1);  R_i = R_{i-1} - g_i (.) B_i (.) h_i
 * for i = 1..K.  The residual is fp32 with one rounding for g_i[r] * h_i[c] and
 * one for the subtraction, so the stored bits are defined exactly.
 * packed:   canonical words, uint32 [K][out][in/32], or NULL.
 * native:   kernel-native tiles (rb_native_bytes(K, out, in) bytes, padding
 *           written as +1), or NULL.  At least one of the two.
 * residual: R_K, fp32 [out][in], or NULL.
 */
int rb_couple(const float *W, const uint16_t *g, const uint16_t *h, int K, int out, int in,
              uint32_t *packed, void *native, float *residual, void *stream);

/*
 * Effective-weight gradient (Eq. RaBiT-grad-wfp), the straight-through gradient
 * of the shared weight: G = (dL/dY) X^T.  Delta fp16 [N][out], X fp16 [N][in],
 * G fp32 [out][in]; fp32 accumulation over the samples in order.  A plain
 * kernel (one thread per element): for large N a dense GEMM library is faster
 * and G may come from there.  out <= 65535.
 */
int rb_weight_grad(const uint16_t *Delta, const uint16_t *X, int N, int out, int in, float *G, void *stream);

/*
 * Gradients of the scales (Eq. RaBiT-grad-gh), binary cores held constant,
 * summed over the samples:
 *   grad_g[i][r] = sum_c B_i[r][c] h_i[c] G[r][c]
 *   grad_h[i][c] = sum_r B_i[r][c] g_i[r] G[r][c]    (the transposed binary product)
 * with G from rb_weight_grad (or any fp32 [out][in] = Delta^T X; 16-byte aligned).  packed:
 * canonical words as rb_couple writes them.  grad_g fp32 [K][out], grad_h fp32
 * [K][in].  workspace: rb_scale_grads_workspace_bytes(K, out, in) bytes, 16-byte
 * aligned (partial column and row sums of the one pass over G that serves both
 * gradients; their order is fixed, results repeat bit for bit).
 */
size_t rb_scale_grads_workspace_bytes(int K, int out, int in);
int rb_scale_grads(const float *G, const uint32_t *packed, const uint16_t *g, const uint16_t *h,
                   int K, int out, int in, float *grad_g, float *grad_h,
                   void *workspace, size_t workspace_bytes, void *stream);

/* ------------------------------------------------------------------------
 * Measurement aids (not part of the layer): the comparators the benchmark
 * reports next to the binary path on the same GPU.
 * ------------------------------------------------------------------------ */

/* Dense fp16 GEMV y = W x with W device fp16 [out][in] row-major, fp32
 * accumulation: the full-precision baseline row of the paper's inference table,
 * hand-written for this GPU.  Requires in % 8 == 0. */
int rb_dense_gemv_f16(const uint16_t *W, const uint16_t *x, uint16_t *y,
                      int out, int in, void *stream);

/* Streams `bytes` (multiple of 16) from device memory with 128-bit loads and
 * writes one 16-byte checksum per workgroup into `sink` (device, at least
 * 16 * rb_stream_read_groups() bytes): the read-bandwidth ceiling of this GPU. */
int rb_stream_read(const void *src, size_t bytes, void *sink, void *stream);
int rb_stream_read_groups(void);

/* Which kernel family the most recent compute call of this thread enqueued:
 * RB_PATH_NONE, RB_PATH_SIGNADD (generic sign-XOR + add kernel, one launch per
 * op), RB_PATH_GEMM (many-token matrix-core GEMM, one launch per op),
 * RB_PATH_MX (matrix-core decode kernels: one layer and token in one launch,
 * or all ops of a stack in one persistent launch) or RB_PATH_BATCH (small-batch
 * kernel of a stack: one pass over the weights for up to 16 tokens, two or
 * three paths, one launch per group of independent ops).  For tests and
 * benchmarks that must know what they measured. */
#define RB_PATH_NONE    0
#define RB_PATH_SIGNADD 1
#define RB_PATH_MX      2
#define RB_PATH_GEMM    3
#define RB_PATH_BATCH   4
int rb_last_path(void);

/* Library version: major*10000 + minor*100 + patch. */
int rb_version(void);

/* ------------------------------------------------------------------------
 * Initialisation of the paths from a full-precision weight (Section 4.3,
 * Alg. 1: Iterative Residual SVID with preconditioning).
 * ------------------------------------------------------------------------ */

/*
 * With W' = row_factors (.) W (.) col_factors (Eq. init-calib; the caller forms
 * the factors (s / max s)^alpha from its channel statistics; NULL means 1):
 *   What_i = 0;  for t = 1..T_max, for i = 1..K:
 *     R_i = W' - sum_{j != i} What_j                            (Eq. init-iter)
 *     B_i = sign(R_i) (sign(0) = +1);  (sigma, a, b) = leading singular triplet of |R_i|
 *     g_i' = sqrt(sigma) a;  h_i' = sqrt(sigma) b;  What_i = g_i' (.) B_i (.) h_i'
 *   g_i = g_i' / row_factors;  h_i = h_i' / col_factors.
 * T_max = 1 is the greedy pass.  fp64 throughout; the triplet comes from a power
 * iteration from the all-ones vector until sigma changes by less than 1e-13
 * relative and b by less than 1e-10 (at most 200 iterations).
 * W fp32 [out][in]; factors fp64 [out], [in]; packed: canonical words, uint32
 * [K][out][in/32]; g fp64 [K][out], h fp64 [K][in]; err: NULL or fp64
 * [T_max][K], the error ||W' - sum_j What_j||_F right after each update.  All
 * device pointers; W, h and col_factors 16-byte aligned (RB_ERR_ALIGN otherwise).
 * workspace: rb_derive_workspace_bytes(out, in) bytes of device memory, 16-byte
 * aligned.  An offline step: it waits for `stream` several times (the
 * host follows the iteration's stopping rule) and has finished when it returns.
 */
size_t rb_derive_workspace_bytes(int out, int in);
int rb_derive_iterative(const float *W, const double *row_factors, const double *col_factors,
                        int K, int T_max, int out, int in,
                        uint32_t *packed, double *g, double *h, double *err,
                        void *workspace, size_t workspace_bytes, void *stream);

/*
 * The decoder block around the layers (the end-to-end decoding setting of
 * Section 5.4 and the inference table: a Llama-2 block), fused into the stack
 * kernel's finishing step so that a whole model's blocks stay one launch.
 * Op n applies layers[layer] to bufs[src] and writes bufs[dst] (device fp16
 * [T][width], as in rb_layer_stack), with
 *   norm >= 0:         the layer reads x / sqrt(mean_j x_j^2 + eps) (.) w with
 *                      w = norm_weights[norm] (device fp16 [in]) in place of x;
 *   RB_EPI_ADD:        dst = y + bufs[aux] (the residual stream; aux may equal dst);
 *   RB_EPI_SILU_MUL:   dst = silu(y) * y_up, y_up = layers[aux] applied to the
 *                      same (normalised) input: the gate and up projections of
 *                      the feed-forward part as one op (same out, in, K);
 * silu(z) = z / (1 + exp(-z)).  Sums, normalisation and epilogues are fp32; only
 * dst is rounded to fp16 (gate and up outputs are never stored).  Ops that share
 * an input and do not depend on each other (q, k, v) run side by side.
 * rb_block_prepare is to a block what rb_stack_prepare is to a plain stack
 * (same rules, may block the host); the prepared ops are run, checked and
 * dropped with rb_stack_run, rb_stack_status and rb_stack_forget.  Two-path
 * layers at T <= 4 or three-path layers at T = 1 (the same number of paths in
 * every layer); RB_ERR_UNSUPPORTED otherwise (run such a block op by op with
 * rb_layer_stack and the three kernels below).  norm_weights is a host array
 * of n_norms device pointers.
 */
#define RB_EPI_NONE 0
#define RB_EPI_ADD 1
#define RB_EPI_SILU_MUL 2
typedef struct rb_block_op { int layer; int src; int dst; int norm; int epilogue; int aux; } rb_block_op;

size_t rb_block_workspace_bytes(const rb_layer *layers, int n_layers, int n_ops, int T);
int rb_block_prepare(const rb_layer *layers, int n_layers,
                     const uint16_t *const *norm_weights, int n_norms, float eps,
                     const rb_block_op *ops, int n_ops,
                     uint16_t *const *bufs, int n_bufs, int T,
                     void *workspace, size_t workspace_bytes, void *stream);
/*
 * The same three operations as kernels of their own (device fp16, fp32
 * arithmetic, one rounding at the end): y[t] = rmsnorm(x[t]) (.) w for T rows
 * of n; y = silu(gate) * up and y = a + b over n elements.  y may be an input.
 */
int rb_rmsnorm(const uint16_t *x, const uint16_t *w, uint16_t *y, int T, int n, float eps, void *stream);
int rb_silu_mul(const uint16_t *gate, const uint16_t *up, uint16_t *y, size_t n, void *stream);
int rb_add(const uint16_t *a, const uint16_t *b, uint16_t *y, size_t n, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* RABIT_H */
