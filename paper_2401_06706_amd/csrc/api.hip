// C ABI of libmcsd: argument validation, error reporting, optional per-kernel
// event timing.  All compute happens in tree_attn.hip, verify_sample.hip, draft_sample.hip and tree_commit.hip.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <mutex>
#include <vector>

#include "mcsd_internal.h"

namespace mcsd {

static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
}

// ------------------------------------------------------------------ event timing
// Off by default.  When on, every kernel launch carries a start and a stop event of its own
// dispatch; mcsd_kernel_timing_read waits for them and adds up the durations.
namespace {
struct EventPair { hipEvent_t a, b; int id; };
std::mutex g_tmutex;
bool g_timing = false;
std::vector<EventPair> g_pending;
double g_total_ms[K_COUNT];
long long g_count[K_COUNT];
const char *const g_names[K_COUNT] = {"tree_attn_mfma", "tree_attn_generic", "tree_attn_combine",
                                      "verify_rows", "walk", "draft_rows", "tree_build", "kv_copy", "kv_finish"};
}  // namespace

bool timing_new_events(hipEvent_t *start, hipEvent_t *stop)
{
    if (!g_timing) return false;
    if (hipEventCreate(start) != hipSuccess) return false;
    if (hipEventCreate(stop) != hipSuccess) { (void)hipEventDestroy(*start); return false; }
    return true;
}

void timing_commit(int id, hipEvent_t start, hipEvent_t stop)
{
    std::lock_guard<std::mutex> lk(g_tmutex);
    g_pending.push_back({start, stop, id});
}

}  // namespace mcsd

using namespace mcsd;

extern "C" {

const char *mcsd_last_error(void) { return g_err; }
const char *mcsd_version(void) { return "libmcsd 0.1 (gfx950)"; }

// Profiling aid (not part of the verification step): enable != 0 starts bracketing
// every kernel launch with HIP events; 0 stops.  Totals are reset when enabled.
int32_t mcsd_kernel_timing(int32_t enable)
{
    std::lock_guard<std::mutex> lk(g_tmutex);
    g_timing = enable != 0;
    if (g_timing) {
        for (auto &p : g_pending) { (void)hipEventDestroy(p.a); (void)hipEventDestroy(p.b); }
        g_pending.clear();
        for (int i = 0; i < K_COUNT; ++i) { g_total_ms[i] = 0.0; g_count[i] = 0; }
    }
    return MCSD_OK;
}

int32_t mcsd_kernel_count(void) { return K_COUNT; }
const char *mcsd_kernel_name(int32_t id) { return (id >= 0 && id < K_COUNT) ? g_names[id] : ""; }

// Waits for the recorded events (synchronises with them) and returns the summed
// duration in ms and the number of launches of kernel `id` since timing was enabled.
int32_t mcsd_kernel_timing_read(int32_t id, double *total_ms, int64_t *launches)
{
    if (id < 0 || id >= K_COUNT || !total_ms || !launches) return MCSD_E_SHAPE;
    std::lock_guard<std::mutex> lk(g_tmutex);
    for (auto &p : g_pending) {
        float ms = 0.f;
        if (hipEventSynchronize(p.b) == hipSuccess && hipEventElapsedTime(&ms, p.a, p.b) == hipSuccess) {
            g_total_ms[p.id] += ms;
            g_count[p.id] += 1;
        }
        (void)hipEventDestroy(p.a);
        (void)hipEventDestroy(p.b);
    }
    g_pending.clear();
    *total_ms = g_total_ms[id];
    *launches = g_count[id];
    return MCSD_OK;
}

int32_t mcsd_tree_validate(const int32_t *parent, int32_t n)
{
    if (!parent) { set_error("parent is NULL"); return MCSD_E_NULL; }
    if (n < 1 || n > MCSD_MAX_NODES) { set_error("n_nodes %d outside 1..%d", n, MCSD_MAX_NODES); return MCSD_E_TREE; }
    for (int i = 0; i < n; ++i)
        if (parent[i] < -1 || parent[i] >= i) {
            set_error("parent[%d] = %d violates -1 <= parent[i] < i", i, parent[i]);
            return MCSD_E_TREE;
        }
    return MCSD_OK;
}

static int32_t check_attn(const mcsd_attn_desc *d, const mcsd_attn_bufs *b, AttnPlan *plan)
{
    if (!d) { set_error("attn desc is NULL"); return MCSD_E_NULL; }
    if (d->struct_size != sizeof(mcsd_attn_desc)) { set_error("attn desc struct_size %u != %zu", d->struct_size, sizeof(mcsd_attn_desc)); return MCSD_E_SHAPE; }
    if (d->B < 1 || d->H_q < 1 || d->H_kv < 1 || d->d < 1 || d->L_stride < 0) { set_error("attn: non-positive size"); return MCSD_E_SHAPE; }
    if (d->L_stride > (1 << 22)) { set_error("attn: L_stride %d > %d", d->L_stride, 1 << 22); return MCSD_E_UNSUPPORTED; }
    if (d->root_row != 0 && d->root_row != 1) { set_error("attn: root_row must be 0 or 1"); return MCSD_E_SHAPE; }
    if (d->N < 1 || d->N + d->root_row > MCSD_MAX_NODES) { set_error("attn: N %d (+ root row) outside 1..%d", d->N, MCSD_MAX_NODES); return MCSD_E_TREE; }
    if (d->H_q % d->H_kv != 0) { set_error("attn: H_q %d not a multiple of H_kv %d", d->H_q, d->H_kv); return MCSD_E_SHAPE; }
    if (d->dtype != MCSD_DTYPE_FP32 && d->dtype != MCSD_DTYPE_BF16) { set_error("attn: unknown dtype %d", d->dtype); return MCSD_E_UNSUPPORTED; }
    if (d->d > MCSD_MAX_HEAD_DIM || d->d % (d->dtype == MCSD_DTYPE_BF16 ? 8 : 4) != 0) { set_error("attn: head dim %d unsupported", d->d); return MCSD_E_UNSUPPORTED; }
    if (!(d->scale >= 0.f) || !(d->scale < 1e30f)) { set_error("attn: scale must be finite and >= 0"); return MCSD_E_SHAPE; }
    if (!make_attn_plan(*d, plan)) { set_error("attn: no kernel for this shape"); return MCSD_E_UNSUPPORTED; }
    if (!b) return MCSD_OK;
    if (b->struct_size != sizeof(mcsd_attn_bufs)) { set_error("attn bufs struct_size %u != %zu", b->struct_size, sizeof(mcsd_attn_bufs)); return MCSD_E_SHAPE; }
    if (!b->q || !b->k_tree || !b->v_tree || !b->prefix_len || !b->parent || !b->out) { set_error("attn: NULL buffer"); return MCSD_E_NULL; }
    if (d->L_stride > 0 && (!b->k_prefix || !b->v_prefix)) { set_error("attn: NULL prefix cache"); return MCSD_E_NULL; }
    if (plan->ws_bytes > 0) {
        if (!b->workspace) { set_error("attn: workspace is NULL, %zu bytes needed", plan->ws_bytes); return MCSD_E_WORKSPACE; }
        if (b->workspace_bytes < plan->ws_bytes) { set_error("attn: workspace %zu < %zu bytes", b->workspace_bytes, plan->ws_bytes); return MCSD_E_WORKSPACE; }
        if (((uintptr_t)b->workspace & 255u) != 0) { set_error("attn: workspace not 256-byte aligned"); return MCSD_E_WORKSPACE; }
    }
    const uintptr_t al = (uintptr_t)b->q | (uintptr_t)b->k_prefix | (uintptr_t)b->v_prefix | (uintptr_t)b->k_tree |
                         (uintptr_t)b->v_tree | (uintptr_t)b->out;
    if (al & 15u) { set_error("attn: tensors must be 16-byte aligned"); return MCSD_E_SHAPE; }
    return MCSD_OK;
}

static int32_t check_verify(const mcsd_verify_desc *d, const mcsd_verify_bufs *b)
{
    if (!d) { set_error("verify desc is NULL"); return MCSD_E_NULL; }
    if (d->struct_size != sizeof(mcsd_verify_desc)) { set_error("verify desc struct_size %u != %zu", d->struct_size, sizeof(mcsd_verify_desc)); return MCSD_E_SHAPE; }
    if (d->B < 1 || d->V < 1 || d->P < 1 || d->gamma_max < 1) { set_error("verify: non-positive size"); return MCSD_E_SHAPE; }
    if (d->N < 1 || d->N > MCSD_MAX_NODES) { set_error("verify: N %d outside 1..%d", d->N, MCSD_MAX_NODES); return MCSD_E_TREE; }
    if (d->P > 1 + d->N) { set_error("verify: P %d > 1+N", d->P); return MCSD_E_SHAPE; }
    if (d->B > 65535) { set_error("verify: B %d > 65535", d->B); return MCSD_E_UNSUPPORTED; }
    if (d->V > MCSD_MAX_VOCAB) { set_error("verify: V %d > %d", d->V, MCSD_MAX_VOCAB); return MCSD_E_UNSUPPORTED; }
    if (d->variant != MCSD_WITH_REPLACEMENT && d->variant != MCSD_WITHOUT_REPLACEMENT && d->variant != MCSD_NAIVE) { set_error("verify: unknown variant %d", d->variant); return MCSD_E_UNSUPPORTED; }
    if (!(d->near_tie_eps >= 0.f)) { set_error("verify: near_tie_eps must be >= 0"); return MCSD_E_SHAPE; }
    if (d->parent_per_seq != 0 && d->parent_per_seq != 1) { set_error("verify: parent_per_seq must be 0 or 1"); return MCSD_E_SHAPE; }
    if (!b) return MCSD_OK;
    if (b->struct_size != sizeof(mcsd_verify_bufs)) { set_error("verify bufs struct_size %u != %zu", b->struct_size, sizeof(mcsd_verify_bufs)); return MCSD_E_SHAPE; }
    if (!b->target_logits || !b->draft_logits || !b->q_row || !b->parent || !b->cand_tok || !b->u_accept ||
        !b->u_endpoint || !b->temperature || !b->n_accepted || !b->accepted_path || !b->out_tokens ||
        !b->acc_child || !b->endpoint || !b->flags) { set_error("verify: NULL buffer"); return MCSD_E_NULL; }
    if (d->V % 4 == 0 && (((uintptr_t)b->target_logits | (uintptr_t)b->draft_logits | (uintptr_t)b->residual_out) & 15u)) {
        set_error("verify: logit arrays must be 16-byte aligned");
        return MCSD_E_SHAPE;
    }
    return MCSD_OK;
}

static int32_t check_draft(const mcsd_draft_desc *d, const mcsd_draft_bufs *b)
{
    if (!d) { set_error("draft desc is NULL"); return MCSD_E_NULL; }
    if (d->struct_size != sizeof(mcsd_draft_desc)) { set_error("draft desc struct_size %u != %zu", d->struct_size, sizeof(mcsd_draft_desc)); return MCSD_E_SHAPE; }
    if (d->B < 1 || d->V < 1 || d->P < 1) { set_error("draft: non-positive size"); return MCSD_E_SHAPE; }
    if (d->N < 1 || d->N > MCSD_MAX_NODES) { set_error("draft: N %d outside 1..%d", d->N, MCSD_MAX_NODES); return MCSD_E_TREE; }
    if (d->P > 1 + d->N) { set_error("draft: P %d > 1+N", d->P); return MCSD_E_SHAPE; }
    if (d->B > 65535) { set_error("draft: B %d > 65535", d->B); return MCSD_E_UNSUPPORTED; }
    if (d->V > MCSD_MAX_VOCAB) { set_error("draft: V %d > %d", d->V, MCSD_MAX_VOCAB); return MCSD_E_UNSUPPORTED; }
    if (d->variant != MCSD_WITH_REPLACEMENT && d->variant != MCSD_WITHOUT_REPLACEMENT) { set_error("draft: unknown variant %d", d->variant); return MCSD_E_UNSUPPORTED; }
    if (!(d->near_tie_eps >= 0.f)) { set_error("draft: near_tie_eps must be >= 0"); return MCSD_E_SHAPE; }
    if (d->parent_per_seq != 0 && d->parent_per_seq != 1) { set_error("draft: parent_per_seq must be 0 or 1"); return MCSD_E_SHAPE; }
    if (!b) { set_error("draft bufs is NULL"); return MCSD_E_NULL; }
    if (b->struct_size != sizeof(mcsd_draft_bufs)) { set_error("draft bufs struct_size %u != %zu", b->struct_size, sizeof(mcsd_draft_bufs)); return MCSD_E_SHAPE; }
    if (!b->draft_logits || !b->q_row || !b->parent || !b->u_draw || !b->temperature || !b->cand_tok || !b->flags) {
        set_error("draft: NULL buffer");
        return MCSD_E_NULL;
    }
    if (d->V % 4 == 0 && ((uintptr_t)b->draft_logits & 15u)) { set_error("draft: draft_logits must be 16-byte aligned"); return MCSD_E_SHAPE; }
    return MCSD_OK;
}

size_t mcsd_attn_workspace_bytes(const mcsd_attn_desc *desc)
{
    AttnPlan plan;
    if (check_attn(desc, nullptr, &plan) != MCSD_OK) return 0;
    return plan.ws_bytes;
}

size_t mcsd_verify_workspace_bytes(const mcsd_verify_desc *desc)
{
    (void)desc;
    return 0;
}

int32_t mcsd_tree_attn(const mcsd_attn_desc *desc, const mcsd_attn_bufs *bufs, void *stream)
{
    AttnPlan plan;
    if (!bufs) { set_error("attn bufs is NULL"); return MCSD_E_NULL; }
    int32_t rc = check_attn(desc, bufs, &plan);
    if (rc != MCSD_OK) return rc;
    return launch_tree_attn(*desc, *bufs, plan, (hipStream_t)stream);
}

// ---------------------------------------------------------- allocation-free attention
// The scratch of mcsd_tree_attn_static lives in the device image of this library: no
// allocation at any call.  In host code the array's name is only a handle for
// hipGetSymbolAddress; the device address it returns (one per GPU) is what kernels get.
static __device__ __align__(256) unsigned char scratch[MCSD_STATIC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[MAX_DEVICES];     // device address of `scratch` on each GPU, looked up once

int32_t static_scratch_of_current_device(void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) { set_error("attn(static): hipGetDevice failed: %s", hipGetErrorString(e)); return MCSD_E_HIP; }
    if (dev < 0 || dev >= MAX_DEVICES) { set_error("attn(static): device %d outside 0..%d", dev, MAX_DEVICES - 1); return MCSD_E_UNSUPPORTED; }
    std::lock_guard<std::mutex> lk(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) {
            set_error("attn(static): hipGetSymbolAddress failed on device %d: %s", dev, hipGetErrorString(e));
            return MCSD_E_HIP;
        }
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return MCSD_OK;
}
}  // namespace

int32_t mcsd_tree_attn_static(const mcsd_attn_desc *desc, const mcsd_attn_bufs *bufs, void *stream)
{
    AttnPlan plan;
    if (!bufs) { set_error("attn bufs is NULL"); return MCSD_E_NULL; }
    int32_t rc = check_attn(desc, nullptr, &plan);       // the descriptor alone fixes the scratch size
    if (rc != MCSD_OK) return rc;
    if (plan.ws_bytes > MCSD_STATIC_SCRATCH_BYTES) {
        set_error("attn(static): this shape needs %zu bytes of scratch, the static buffer holds %zu; use mcsd_tree_attn with a workspace",
                  plan.ws_bytes, (size_t)MCSD_STATIC_SCRATCH_BYTES);
        return MCSD_E_WORKSPACE;
    }
    if (bufs->struct_size != sizeof(mcsd_attn_bufs)) { set_error("attn bufs struct_size %u != %zu", bufs->struct_size, sizeof(mcsd_attn_bufs)); return MCSD_E_SHAPE; }
    mcsd_attn_bufs b = *bufs;
    void *ptr = nullptr;
    rc = static_scratch_of_current_device(&ptr);
    if (rc != MCSD_OK) return rc;
    b.workspace = ptr;
    b.workspace_bytes = MCSD_STATIC_SCRATCH_BYTES;
    rc = check_attn(desc, &b, &plan);
    if (rc != MCSD_OK) return rc;
    return launch_tree_attn(*desc, b, plan, (hipStream_t)stream);
}

int32_t mcsd_tree_attn_paged(const mcsd_attn_desc *desc, const mcsd_attn_bufs *bufs, const mcsd_paged_kv *paged,
                             void *stream)
{
    AttnPlan plan;
    if (!bufs) { set_error("attn bufs is NULL"); return MCSD_E_NULL; }
    if (!paged) { set_error("paged descriptor is NULL"); return MCSD_E_NULL; }
    int32_t rc = check_attn(desc, bufs, &plan);
    if (rc != MCSD_OK) return rc;
    if (paged->struct_size != sizeof(mcsd_paged_kv)) { set_error("paged struct_size %u != %zu", paged->struct_size, sizeof(mcsd_paged_kv)); return MCSD_E_SHAPE; }
    if (!paged->block_table) { set_error("paged: block_table is NULL"); return MCSD_E_NULL; }
    if (paged->page_size < 32 || paged->page_size % 32 != 0) { set_error("paged: page_size %d is not a positive multiple of 32", paged->page_size); return MCSD_E_SHAPE; }
    if (paged->n_pages < 1 || paged->max_pages_per_seq < 1) { set_error("paged: non-positive size"); return MCSD_E_SHAPE; }
    if ((long)paged->max_pages_per_seq * paged->page_size < (long)desc->L_stride) { set_error("paged: L_stride %d exceeds max_pages_per_seq * page_size", desc->L_stride); return MCSD_E_SHAPE; }
    return launch_tree_attn(*desc, *bufs, plan, (hipStream_t)stream, paged);
}

int32_t mcsd_verify_sample(const mcsd_verify_desc *desc, const mcsd_verify_bufs *bufs, void *stream)
{
    if (!bufs) { set_error("verify bufs is NULL"); return MCSD_E_NULL; }
    int32_t rc = check_verify(desc, bufs);
    if (rc != MCSD_OK) return rc;
    return launch_verify(*desc, *bufs, (hipStream_t)stream);
}

int32_t mcsd_draft_sample(const mcsd_draft_desc *desc, const mcsd_draft_bufs *bufs, void *stream)
{
    int32_t rc = check_draft(desc, bufs);
    if (rc != MCSD_OK) return rc;
    return launch_draft_sample(*desc, *bufs, (hipStream_t)stream);
}

int32_t mcsd_tree_size(const int32_t *kconfig, int32_t gamma, int32_t *n_nodes, int32_t *n_draft_rows)
{
    if (!kconfig) { set_error("tree: kconfig is NULL"); return MCSD_E_NULL; }
    if (gamma < 1 || gamma > MAX_GAMMA) { set_error("tree: gamma %d outside 1..%d", gamma, MAX_GAMMA); return MCSD_E_SHAPE; }
    long level = 1, n = 0, internal = 1;
    for (int i = 0; i < gamma; ++i) {
        if (kconfig[i] < 1) { set_error("tree: k_%d = %d < 1", i + 1, kconfig[i]); return MCSD_E_SHAPE; }
        level *= kconfig[i];
        n += level;
        if (n > MCSD_MAX_NODES) { set_error("tree: more than %d nodes", MCSD_MAX_NODES); return MCSD_E_TREE; }
        if (i + 1 < gamma) internal += level;
    }
    if (n_nodes) *n_nodes = (int32_t)n;
    if (n_draft_rows) *n_draft_rows = (int32_t)internal;
    return MCSD_OK;
}

int32_t mcsd_tree_build(const int32_t *kconfig, int32_t gamma, int32_t B, const int32_t *prefix_len, int32_t *parent,
                        int32_t *depth, int32_t *q_row, int32_t *position_ids, int32_t root_row, void *stream)
{
    if (root_row != 0 && root_row != 1) { set_error("tree: root_row must be 0 or 1"); return MCSD_E_SHAPE; }
    int32_t n = 0;
    int32_t rc = mcsd_tree_size(kconfig, gamma, &n, nullptr);
    if (rc != MCSD_OK) return rc;
    if (!parent || !depth || !q_row) { set_error("tree: NULL output"); return MCSD_E_NULL; }
    if (position_ids && !prefix_len) { set_error("tree: position_ids needs prefix_len"); return MCSD_E_NULL; }
    if (position_ids && (B < 1 || B > 65535)) { set_error("tree: B %d outside 1..65535", B); return MCSD_E_SHAPE; }
    return launch_tree_build(kconfig, gamma, n, B, prefix_len, parent, depth, q_row, position_ids, root_row, (hipStream_t)stream);
}

static int32_t check_commit(const mcsd_commit_desc *d, const mcsd_commit_bufs *b)
{
    if (!d) { set_error("commit desc is NULL"); return MCSD_E_NULL; }
    if (d->struct_size != sizeof(mcsd_commit_desc)) { set_error("commit desc struct_size %u != %zu", d->struct_size, sizeof(mcsd_commit_desc)); return MCSD_E_SHAPE; }
    if (d->B < 1 || d->H_kv < 1 || d->d < 1 || d->L_stride < 1 || d->gamma_max < 1 || d->n_layers < 1) { set_error("commit: non-positive size"); return MCSD_E_SHAPE; }
    if (d->root_row != 0 && d->root_row != 1) { set_error("commit: root_row must be 0 or 1"); return MCSD_E_SHAPE; }
    if (d->N < 1 || d->N + d->root_row > MCSD_MAX_NODES) { set_error("commit: N %d (+ root row) outside 1..%d", d->N, MCSD_MAX_NODES); return MCSD_E_TREE; }
    if (d->dtype != MCSD_DTYPE_FP32 && d->dtype != MCSD_DTYPE_BF16) { set_error("commit: unknown dtype %d", d->dtype); return MCSD_E_UNSUPPORTED; }
    const int esize = d->dtype == MCSD_DTYPE_FP32 ? 4 : 2;
    if ((d->d * esize) % 16 != 0) { set_error("commit: d * element size must be a multiple of 16 bytes"); return MCSD_E_SHAPE; }
    if (d->B > 65535 || d->gamma_max > 65535 || d->n_layers > 65535) { set_error("commit: grid too large"); return MCSD_E_UNSUPPORTED; }
    if (!b) { set_error("commit bufs is NULL"); return MCSD_E_NULL; }
    if (b->struct_size != sizeof(mcsd_commit_bufs)) { set_error("commit bufs struct_size %u != %zu", b->struct_size, sizeof(mcsd_commit_bufs)); return MCSD_E_SHAPE; }
    if (!b->k_prefix || !b->v_prefix || !b->k_tree || !b->v_tree || !b->n_accepted || !b->accepted_path ||
        !b->out_tokens || !b->prefix_len || !b->next_root || !b->flags) { set_error("commit: NULL buffer"); return MCSD_E_NULL; }
    if (((uintptr_t)b->k_prefix | (uintptr_t)b->v_prefix | (uintptr_t)b->k_tree | (uintptr_t)b->v_tree) & 15u) {
        set_error("commit: caches must be 16-byte aligned");
        return MCSD_E_SHAPE;
    }
    return MCSD_OK;
}

int32_t mcsd_kv_commit(const mcsd_commit_desc *d, const mcsd_commit_bufs *b, void *stream)
{
    const int32_t rc = check_commit(d, b);
    if (rc != MCSD_OK) return rc;
    return launch_kv_commit(*d, *b, (hipStream_t)stream);
}

int32_t mcsd_kv_commit_paged(const mcsd_commit_desc *d, const mcsd_commit_bufs *b, const mcsd_paged_kv *paged, void *stream)
{
    int32_t rc = check_commit(d, b);
    if (rc != MCSD_OK) return rc;
    if (!paged) { set_error("paged descriptor is NULL"); return MCSD_E_NULL; }
    if (paged->struct_size != sizeof(mcsd_paged_kv)) { set_error("paged struct_size %u != %zu", paged->struct_size, sizeof(mcsd_paged_kv)); return MCSD_E_SHAPE; }
    if (!paged->block_table) { set_error("paged: block_table is NULL"); return MCSD_E_NULL; }
    if (paged->page_size < 32 || paged->page_size % 32 != 0) { set_error("paged: page_size %d is not a positive multiple of 32", paged->page_size); return MCSD_E_SHAPE; }
    if (paged->n_pages < 1 || paged->max_pages_per_seq < 1) { set_error("paged: non-positive size"); return MCSD_E_SHAPE; }
    if ((long)paged->max_pages_per_seq * paged->page_size < (long)d->L_stride) { set_error("paged: L_stride %d exceeds max_pages_per_seq * page_size", d->L_stride); return MCSD_E_SHAPE; }
    return launch_kv_commit(*d, *b, (hipStream_t)stream, paged);
}

int32_t mcsd_verify_step(const mcsd_attn_desc *ad, const mcsd_attn_bufs *ab, const mcsd_verify_desc *vd,
                         const mcsd_verify_bufs *vb, void *stream)
{
    AttnPlan plan;
    if (!ab || !vb) { set_error("bufs is NULL"); return MCSD_E_NULL; }
    int32_t rc = check_attn(ad, ab, &plan);
    if (rc != MCSD_OK) return rc;
    rc = check_verify(vd, vb);
    if (rc != MCSD_OK) return rc;
    // The merge of the attention partials and the walk are the two small tail kernels of the step;
    // when the attention is split they go out as one launch after the verification rows, and when
    // it is not, the walk rides on the attention launch, which then follows the verification rows.
    if (plan.use_mfma && plan.n_chunks_max > 1) {
        rc = launch_tree_attn(*ad, *ab, plan, (hipStream_t)stream, nullptr, ATTN_PHASE_MAIN);
        if (rc != MCSD_OK) return rc;
        rc = launch_verify(*vd, *vb, (hipStream_t)stream, false);
        if (rc != MCSD_OK) return rc;
        const WalkParams w = make_walk_params(*vd, *vb);
        return launch_tree_attn(*ad, *ab, plan, (hipStream_t)stream, nullptr, ATTN_PHASE_COMBINE, &w);
    }
    if (plan.use_mfma) {
        // no merge launch: the verification rows go first and the attention launch carries the walk
        rc = launch_verify(*vd, *vb, (hipStream_t)stream, false);
        if (rc != MCSD_OK) return rc;
        const WalkParams w = make_walk_params(*vd, *vb);
        return launch_tree_attn(*ad, *ab, plan, (hipStream_t)stream, nullptr, ATTN_PHASE_MAIN, &w);
    }
    rc = launch_tree_attn(*ad, *ab, plan, (hipStream_t)stream);
    if (rc != MCSD_OK) return rc;
    return launch_verify(*vd, *vb, (hipStream_t)stream);
}

int32_t mcsd_attn_plan_override(int32_t variant, int32_t chunk_tiles, int32_t target_items)
{
    const int32_t rc = attn_plan_override(variant, chunk_tiles, target_items);
    if (rc != MCSD_OK) set_error("plan override: variant must be 0..3, chunk_tiles and target_items >= 0");
    return rc;
}

}  // extern "C"
