// Kernel selection for one layer and for a stack of layers.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <map>
#include <mutex>
#include <vector>

#include "rabit.h"
#include "rb_internal.h"

namespace rb {

thread_local int g_last_path = RB_PATH_NONE;
void set_last_path(int path) { g_last_path = path; }

// The fused decode kernel takes up to four tokens per launch.  A two-path stack of 5 to
// BATCH_MIN_T - 1 tokens runs as passes of that kernel over consecutive groups of four tokens (the
// last pass takes what is left): one pass is one launch for the whole op list.
constexpr int PASS_T = 4;
constexpr int PAIRS_MAX_T = 16;

static size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
// one slot per pass, sized for the largest plan any pass may hold (a one-token plan has longer step
// lists than a four-token one: more compute wavefronts)
static size_t pair_stride(const rb_layer *layers, int n_layers, int n_ops)
{
    size_t need = 0;
    for (int t = 1; t <= PASS_T; ++t) need = std::max(need, mx::plan_workspace_bytes(layers, n_layers, n_ops, t));
    return round_up(need, 256);
}
static bool pairs_apply(const rb_layer *layers, int n_layers, int n_ops, int T)
{
    if (n_ops < 2 || T <= PASS_T || T > PAIRS_MAX_T) return false;
    for (int l = 0; l < n_layers; ++l)
        if (layers[l].K != 2 || !mx::layer_supported(&layers[l], PASS_T) || layers[l].out % 8 != 0) return false;   // rows of a pass stay 16-byte aligned
    return true;
}

// Which stacks take the small-batch kernel (one pass over the weights for all tokens): every stack
// with a three-path layer, and two-path stacks of BATCH_MIN_T tokens or more.  Below that the passes
// over groups of four tokens on the fused decode kernel are faster (measured on the 7B-shaped
// dependent chain: 1.3 ms for one pass at 4 tokens against 2.1 ms; 2.2 ms for two passes at 6;
// 2.7 against 2.5 ms at 8): the small-batch kernel is one launch per group of independent ops, and
// a launch of a few hundred KB per workgroup is bound by memory latency, not by the bytes it streams.
constexpr int BATCH_MIN_T = 8;
bool batch_applies(const rb_layer *layers, int n_layers, int T)
{
    bool any_three = false, all_three = true;
    for (int l = 0; l < n_layers; ++l) {
        if (!batch::layer_supported(&layers[l], T)) return false;
        any_three = any_three || layers[l].K == 3;
        all_three = all_three && layers[l].K == 3;
    }
    if (all_three && T == 1) return false;       // one token, three paths throughout: the fused decode kernel
    return any_three || T >= BATCH_MIN_T;
}

static bool batch_supported(const rb_layer *layers, int n_layers, int T)
{
    for (int l = 0; l < n_layers; ++l)
        if (!batch::layer_supported(&layers[l], T)) return false;
    return true;
}

// A single call on a three-path layer reads the weights once from K3_ONE_PASS_MIN_T tokens on: the
// small-batch kernel as a plan of one op up to K3_BATCH_MAX_T fp16 tokens, the many-token kernel
// beyond that and for other element types.  Below, the generic kernel's one launch (its passes
// over the weights, one per token, come out of the caches) beats their four or five.  Measured per
// call at 4096x4096 / 11008x4096 / 4096x11008: generic 26 / 52 / 64 us at 4 tokens, 43 / 95 / 99
// at 8, 76 / 175 / 188 at 16; small-batch 38 / 38 / 66, 46 / 47 / 86, 60 / 61 / 124; many-token
// 57 / 58 / 111 whatever the count.
constexpr int K3_ONE_PASS_MIN_T = 6, K3_BATCH_MAX_T = 12;
static bool single_batch_applies(const rb_layer *L, int T)
{
    return L->K == 3 && T >= K3_ONE_PASS_MIN_T && T <= K3_BATCH_MAX_T && batch::layer_supported(L, T);
}
bool single_gemm_applies(const rb_layer *L, int T)
{
    return T > 2 && (L->K != 3 || T >= K3_ONE_PASS_MIN_T) && gemm::supported(L, T);
}

size_t workspace_bytes(const rb_layer *layers, int n_layers, int n_ops, int T)
{
    // one layer, one token: the single-call kernel keeps everything in LDS
    if (n_layers == 1 && n_ops == 1 && T == 1 && gemv1::supported(&layers[0], 1)) return 0;
    // one three-path layer at a few tokens: the small-batch kernel as a plan of one op; other
    // element types than fp16 in and out: the many-token kernel
    if (n_layers == 1 && n_ops == 1 && single_batch_applies(&layers[0], T))
        return std::max(batch::plan_workspace_bytes(layers, 1, 1, T), gemm::workspace_bytes(&layers[0], T));
    if (batch_applies(layers, n_layers, T) && n_ops > 1) {
        size_t need = batch::plan_workspace_bytes(layers, n_layers, n_ops, T);
        // the ops of a stack the kernel turns down run one after the other on the general paths
        for (int l = 0; l < n_layers; ++l)
            if (T > 2 && gemm::supported(&layers[l], T)) need = std::max(need, gemm::workspace_bytes(&layers[l], T));
        return need;
    }
    if (T > PASS_T) {
        // ops run one after the other on the caller's stream and share the scratch of the GEMM path
        size_t need = 0;
        for (int l = 0; l < n_layers; ++l)
            if (gemm::supported(&layers[l], T)) need = need > gemm::workspace_bytes(&layers[l], T) ? need : gemm::workspace_bytes(&layers[l], T);
        if (pairs_apply(layers, n_layers, n_ops, T)) {
            const size_t pairs = (size_t)((T + PASS_T - 1) / PASS_T) * pair_stride(layers, n_layers, n_ops);
            need = need > pairs ? need : pairs;
        }
        // rb_layer_stack takes the small-batch kernel rather than set up several passes
        if (n_ops > 1 && batch_supported(layers, n_layers, T))
            need = std::max(need, batch::plan_workspace_bytes(layers, n_layers, n_ops, T));
        return need;
    }
    size_t need = mx::plan_workspace_bytes(layers, n_layers, n_ops, T);
    // three or four tokens: a single call (and whatever the fused kernel turns down) takes the many-token kernel
    for (int l = 0; l < n_layers && T > 2; ++l)
        if (gemm::supported(&layers[l], T)) need = std::max(need, gemm::workspace_bytes(&layers[l], T));
    return need;
}

// host record of a workspace that holds one plan per pass
struct PairPlans { int passes; size_t stride; };
static std::mutex g_pairs_mutex;
static std::map<const void *, PairPlans> g_pairs;

int prepare_pairs(const rb_layer *layers, int n_layers, const rb_stack_op *ops, int n_ops, uint16_t *const *bufs,
                  int n_bufs, int T, void *workspace, size_t workspace_bytes_, hipStream_t stream)
{
    if (!pairs_apply(layers, n_layers, n_ops, T)) return RB_ERR_UNSUPPORTED;
    const size_t stride = pair_stride(layers, n_layers, n_ops);
    const int passes = (T + PASS_T - 1) / PASS_T;
    if (!workspace || workspace_bytes_ < stride * (size_t)passes) return RB_ERR_WORKSPACE;
    // width of every buffer an op touches
    std::vector<int> width((size_t)n_bufs, 0);
    for (int n = 0; n < n_ops; ++n) {
        const rb_layer &L = layers[ops[n].layer];
        int &ws = width[(size_t)ops[n].src], &wd = width[(size_t)ops[n].dst];
        if ((ws && ws != L.in) || (wd && wd != L.out)) return RB_ERR_SHAPE;
        ws = L.in;
        wd = L.out;
    }
    std::vector<uint16_t *> sub((size_t)n_bufs);
    for (int p = 0; p < passes; ++p) {
        for (int b = 0; b < n_bufs; ++b) sub[(size_t)b] = bufs[b] ? bufs[b] + (size_t)p * PASS_T * (size_t)width[(size_t)b] : nullptr;
        const int rc = mx::prepare_plan(layers, ops, n_ops, sub.data(), std::min(PASS_T, T - p * PASS_T),
                                        static_cast<uint8_t *>(workspace) + (size_t)p * stride, stride, stream);
        if (rc != RB_OK) {
            // drop the records of the passes already prepared: the workspace holds no usable stack
            for (int q = 0; q < p; ++q) mx::forget_plan(static_cast<uint8_t *>(workspace) + (size_t)q * stride);
            return rc;
        }
    }
    std::lock_guard<std::mutex> lock(g_pairs_mutex);
    g_pairs[workspace] = PairPlans{passes, stride};
    return RB_OK;
}

// RB_ERR_UNSUPPORTED: the workspace holds no plans of this kind
int run_pairs(void *workspace, size_t workspace_bytes_, hipStream_t stream)
{
    PairPlans pp;
    {
        std::lock_guard<std::mutex> lock(g_pairs_mutex);
        const auto it = g_pairs.find(workspace);
        if (it == g_pairs.end()) return RB_ERR_UNSUPPORTED;
        pp = it->second;
    }
    if (workspace_bytes_ < pp.stride * (size_t)pp.passes) return RB_ERR_WORKSPACE;
    for (int p = 0; p < pp.passes; ++p) {
        const int rc = mx::launch_plan(static_cast<uint8_t *>(workspace) + (size_t)p * pp.stride, pp.stride, stream);
        if (rc != RB_OK) return rc;
    }
    return RB_OK;
}

int pairs_status(const void *workspace, hipStream_t stream, unsigned long long *waited, int *reason)
{
    PairPlans pp;
    {
        std::lock_guard<std::mutex> lock(g_pairs_mutex);
        const auto it = g_pairs.find(workspace);
        if (it == g_pairs.end()) return RB_ERR_UNSUPPORTED;
        pp = it->second;
    }
    for (int p = 0; p < pp.passes; ++p) {
        const int rc = mx::plan_status(static_cast<const uint8_t *>(workspace) + (size_t)p * pp.stride, stream, waited, reason);
        if (rc != RB_OK) return rc;
    }
    return RB_OK;
}

void forget_pairs(const void *workspace)
{
    PairPlans pp{0, 0};
    {
        std::lock_guard<std::mutex> lock(g_pairs_mutex);
        const auto it = g_pairs.find(workspace);
        if (it == g_pairs.end()) return;
        pp = it->second;
        g_pairs.erase(it);
    }
    for (int p = 0; p < pp.passes; ++p) mx::forget_plan(static_cast<const uint8_t *>(workspace) + (size_t)p * pp.stride);
}

int dispatch_linear(const rb_layer *L, const void *X, void *Y, int T, int act_dtype, int out_dtype,
                    void *workspace, size_t workspace_bytes, hipStream_t stream)
{
    if (act_dtype == RB_F16 && out_dtype == RB_F16 && gemv1::supported(L, T)) {
        g_last_path = RB_PATH_MX;
        return gemv1::launch(L, X, Y, stream);
    }
    if (act_dtype == RB_F16 && out_dtype == RB_F16 && L->K == 2 && T <= 2 && mx::layer_supported(L, T) && workspace &&
        workspace_bytes >= mx::plan_workspace_bytes(L, 1, 1, T)) {
        const rb_stack_op op{0, 0, 1};
        uint16_t *bufs[2] = {static_cast<uint16_t *>(const_cast<void *>(X)), static_cast<uint16_t *>(Y)};
        batch::forget_plan(workspace);
        const int rc = mx::run_plan(L, &op, 1, bufs, T, workspace, workspace_bytes, stream);
        if (rc != RB_ERR_UNSUPPORTED) { g_last_path = RB_PATH_MX; return rc; }
    }
    if (act_dtype == RB_F16 && out_dtype == RB_F16 && single_batch_applies(L, T) && workspace &&
        workspace_bytes >= batch::plan_workspace_bytes(L, 1, 1, T)) {
        const rb_stack_op op{0, 0, 1};
        uint16_t *bufs[2] = {static_cast<uint16_t *>(const_cast<void *>(X)), static_cast<uint16_t *>(Y)};
        int rc = batch::prepare_plan(L, &op, 1, bufs, T, workspace, workspace_bytes, stream);
        if (rc == RB_OK) rc = batch::launch_plan(workspace, workspace_bytes, stream);
        if (rc != RB_ERR_UNSUPPORTED) { g_last_path = RB_PATH_BATCH; return rc; }
    }
    if (single_gemm_applies(L, T) && workspace && workspace_bytes >= gemm::workspace_bytes(L, T)) {
        g_last_path = RB_PATH_GEMM;
        return gemm::launch(L, X, Y, T, act_dtype, out_dtype, workspace, stream);
    }
    g_last_path = RB_PATH_SIGNADD;
    return launch_signadd(L, X, Y, T, act_dtype, out_dtype, stream);
}

int dispatch_stack(const rb_layer *layers, int n_layers, const rb_stack_op *ops, int n_ops,
                   uint16_t *const *bufs, int n_bufs, int T, void *workspace, size_t workspace_bytes, hipStream_t stream)
{
    if (n_ops > 1 && (batch_applies(layers, n_layers, T) || (T > PASS_T && batch_supported(layers, n_layers, T)))) {
        int rc = batch::prepare_plan(layers, ops, n_ops, bufs, T, workspace, workspace_bytes, stream);
        if (rc == RB_OK) rc = batch::launch_plan(workspace, workspace_bytes, stream);
        if (rc == RB_OK) g_last_path = RB_PATH_BATCH;
        if (rc != RB_ERR_UNSUPPORTED && rc != RB_ERR_WORKSPACE) return rc;
    }
    bool fused = workspace && workspace_bytes >= mx::plan_workspace_bytes(layers, n_layers, n_ops, T);
    for (int n = 0; n < n_ops && fused; ++n) fused = mx::layer_supported(&layers[ops[n].layer], T);
    if (fused) {
        batch::forget_plan(workspace);
        const int rc = mx::run_plan(layers, ops, n_ops, bufs, T, workspace, workspace_bytes, stream);
        if (rc != RB_ERR_UNSUPPORTED) { g_last_path = RB_PATH_MX; return rc; }
    }
    for (int n = 0; n < n_ops; ++n) {
        const rb_layer *L = &layers[ops[n].layer];
        const int rc = dispatch_linear(L, bufs[ops[n].src], bufs[ops[n].dst], T, RB_F16, RB_F16, workspace,
                                       workspace_bytes, stream);
        if (rc != RB_OK) return rc;
    }
    return RB_OK;
}

}  // namespace rb

extern "C" int rb_last_path(void) { return rb::g_last_path; }
