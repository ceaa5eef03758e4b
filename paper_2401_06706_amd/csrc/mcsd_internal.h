// Internal declarations shared by the translation units of libmcsd (HIP, gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "mcsd.h"

namespace mcsd {

// Kernel ids for the optional per-kernel event timing.
enum KernelId { K_ATTN_MFMA = 0, K_ATTN_GENERIC = 1, K_ATTN_COMBINE = 2, K_VERIFY_ROWS = 3, K_WALK = 4, K_DRAFT_ROWS = 5, K_TREE_BUILD = 6, K_KV_COPY = 7, K_KV_FINISH = 8, K_COUNT = 9 };

void set_error(const char *fmt, ...);

// Optional per-kernel timing.  When it is enabled a launch goes out through the HIP extension
// that ties a start and a stop event to that one dispatch, so the elapsed time between them is
// the kernel's own execution time (what a kernel trace reports), not launch latency or gaps.
bool timing_new_events(hipEvent_t *start, hipEvent_t *stop);        // false: timing is off
void timing_commit(int kernel_id, hipEvent_t start, hipEvent_t stop);

template <typename Kernel, typename... Args>
inline void launch_kernel(int kernel_id, Kernel kernel, dim3 grid, dim3 block, hipStream_t stream, Args... args)
{
    hipEvent_t e0, e1;
    if (timing_new_events(&e0, &e1)) {
        hipExtLaunchKernelGGL(kernel, grid, block, 0, stream, e0, e1, 0, args...);
        timing_commit(kernel_id, e0, e1);
    } else {
        hipLaunchKernelGGL(kernel, grid, block, 0, stream, args...);
    }
}

// ---- the walk (Sec. 3), shared by verify_sample.hip and the fused tail of a step -------
struct WalkParams {
    int B, N, gamma_max;
    const int32_t *acc_child, *endpoint, *cand_tok;
    int32_t *n_accepted, *accepted_path, *out_tokens;
    uint32_t *flags;        // [B][1+N], written by the verification rows before the walk runs
};

// From the root: an accepted child moves down one level, otherwise (or at a leaf) the row's
// endpoint closes the block.
__device__ __forceinline__ void walk_sequence(const WalkParams &w, int b)
{
    const int N = w.N, G = w.gamma_max;
    int32_t *path = w.accepted_path + (size_t)b * G;
    int32_t *out = w.out_tokens + (size_t)b * (G + 1);
    for (int i = 0; i < G; ++i) path[i] = -1;
    for (int i = 0; i <= G; ++i) out[i] = -1;
    int row = 0, n = 0;
    for (;;) {
        const size_t rix = (size_t)b * (1 + N) + row;
        const int c = w.acc_child[rix];
        if (c < 0 || c >= N || n >= G) {
            // A row that accepted a child has no endpoint: reaching gamma_max there means the tree
            // is deeper than the caller said (the block then ends with -1 and the row is flagged).
            if (c >= 0 && c < N) atomicOr(&w.flags[rix], (uint32_t)MCSD_FLAG_BAD_TREE);
            out[n] = w.endpoint[rix];
            break;
        }
        path[n] = c;
        out[n] = w.cand_tok[(size_t)b * N + c];
        ++n;
        row = 1 + c;
    }
    w.n_accepted[b] = n;
}

// ---- tree attention -------------------------------------------------------
struct AttnPlan {
    bool use_mfma;        // bf16, d == 128: matrix-core kernel; otherwise the generic ALU kernel
    int rows_per_kv;      // M = N * (H_q / H_kv) query rows that share one KV head
    int row_tile;         // query rows per workgroup (32 or 64) for the MFMA kernel
    int variant;          // which instantiation of the MFMA kernel
    int n_row_tiles;
    int tiles_prefix_max; // 32-key tiles needed for L_stride prefix keys
    int tiles_tree;       // 32-key tiles needed for N tree keys
    int chunk_tiles;      // 32-key tiles per workgroup
    int n_chunks_max;     // grid extent along the key axis
    size_t partial_stride_rows; // rows per (b, g) in the partial buffers = n_row_tiles * row_tile
    size_t ws_bytes;
};

bool make_attn_plan(const mcsd_attn_desc &d, AttnPlan *plan);
// Process-wide overrides of the plan (0 = automatic): kernel variant 1..3, 32-key tiles per
// segment, workgroups aimed at when the segment length is derived.  A test and tuning aid.
int32_t attn_plan_override(int variant, int chunk_tiles, int target_wgs);
// phases: the attention kernel, and the merge of the split partials (needed iff
// plan.n_chunks_max > 1).  The last launch of the attention (the merge, or the matrix-core
// kernel itself when nothing is split) can carry the walk of a verification that ran before
// it on the same stream (tail_walk), which saves a step one kernel launch.
enum { ATTN_PHASE_MAIN = 1, ATTN_PHASE_COMBINE = 2, ATTN_PHASE_ALL = 3 };
int32_t launch_tree_attn(const mcsd_attn_desc &d, const mcsd_attn_bufs &b, const AttnPlan &plan,
                         hipStream_t stream, const mcsd_paged_kv *paged = nullptr, int phases = ATTN_PHASE_ALL,
                         const WalkParams *tail_walk = nullptr);

// ---- verification ---------------------------------------------------------
int32_t launch_verify(const mcsd_verify_desc &d, const mcsd_verify_bufs &b, hipStream_t stream, bool with_walk = true);
WalkParams make_walk_params(const mcsd_verify_desc &d, const mcsd_verify_bufs &b);

// ---- draft-side candidates ------------------------------------------------
int32_t launch_draft_sample(const mcsd_draft_desc &d, const mcsd_draft_bufs &b, hipStream_t stream);

// ---- candidate tree and KV commit -----------------------------------------
constexpr int MAX_GAMMA = 16;
int32_t launch_tree_build(const int32_t *kconfig, int gamma, int n_nodes, int B, const int32_t *prefix_len,
                          int32_t *parent, int32_t *depth, int32_t *q_row, int32_t *position_ids, int root_row, hipStream_t stream);
int32_t launch_kv_commit(const mcsd_commit_desc &d, const mcsd_commit_bufs &b, hipStream_t stream,
                         const mcsd_paged_kv *paged = nullptr);

}  // namespace mcsd
