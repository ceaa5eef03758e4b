/*
 * mcsd.h - C ABI of libmcsd: the target-side verification step of
 * Multi-Candidate Speculative Decoding (MCSD) on one AMD MI355X (gfx950).
 *
 * Operations, all enqueued asynchronously on a caller-supplied HIP stream:
 *
 *   mcsd_tree_attn      Tree attention (Sec. 3.3 of the paper): all candidate
 *                       tokens of the draft tree are scored in one pass against
 *                       the shared prefix KV cache; a candidate attends to the
 *                       whole prefix, to its ancestors in the tree and to itself.
 *   mcsd_verify_sample  Multi-candidate speculative sampling, Algorithm 1 (with
 *                       replacement) and Algorithm 2 (without replacement), run
 *                       for every node that has children, the endpoint draws of
 *                       Sec. 2 / Sec. 3, and the root-to-leaf walk of Sec. 3 that
 *                       turns the per-node outcomes into the accepted path.
 *   mcsd_verify_step    Both, back to back on one stream: one layer's tree
 *                       attention followed by one verification.
 *   mcsd_draft_sample   The step before: the k candidates of every parent drawn
 *                       from the draft distribution (Sec. 3.1; Eq. (1) when
 *                       sampling without replacement).
 *   mcsd_tree_build     The candidate tree of a k-configuration (parent, depth,
 *                       draft-row map, position ids) built on the device.
 *   mcsd_kv_commit      The step after: the accepted path's keys and values join
 *                       the prefix cache, prefix_len grows, the endpoint becomes
 *                       the next root.
 *
 * Conventions
 *   - Plain C, plain-old-data structs; the first field of every struct is its
 *     own size in bytes (set it with sizeof) so the layout can be versioned.
 *   - Every data pointer in a *_bufs struct is a DEVICE pointer that the caller
 *     owns; the library never allocates, frees or keeps device memory.  Scratch
 *     space comes in through `workspace` (size from mcsd_*_workspace_bytes) and
 *     may be reused by the caller as soon as the stream has passed the call.
 *     Descriptor structs and the arguments of mcsd_tree_validate are HOST memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls return after enqueueing; outputs are valid once the stream is
 *     synchronised.  Two calls that share a workspace must be stream-ordered.
 *   - Return value: MCSD_OK or a negative MCSD_E_* code.  Every argument is
 *     validated before the first launch: on an argument error (every code but
 *     MCSD_E_HIP) nothing has been enqueued.  MCSD_E_HIP means the HIP runtime
 *     refused a launch; launches enqueued before it stay enqueued and the
 *     outputs of the call are undefined.  mcsd_last_error() gives a thread-local
 *     message.  No call aborts, throws or synchronises the device.
 *   - Errors in the DATA (token id out of range, zero draft probability, ...)
 *     cannot be seen from the host without a sync; they set bits in the
 *     `flags` output instead (MCSD_FLAG_*).
 *   - Tree layout: nodes 0..N-1 exclude the root.  parent[i] == -1 marks a child of the
 *     root; parent[i] < i is required (any order in which parents precede
 *     children, e.g. generation order).  The children of a node are verified
 *     in ascending node id, which must be the order they were sampled in
 *     (Algorithm 2 depends on it).  "Row" r means the root for r == 0 and node
 *     r-1 otherwise.  N <= MCSD_MAX_NODES.
 *   - The root and the caches.  By default (root_row = 0) the root is the last token of
 *     the context and its keys and values are already in the prefix cache: it is neither a
 *     query nor a key row of the tree block, which is the situation of one verification
 *     step looked at alone.  In a decode loop the root of a step is the endpoint token the
 *     previous step emitted, and the target's forward pass over "root + candidates"
 *     produces the root's keys and values together with the candidates' (its logit row
 *     is row 0 of target_logits).  root_row = 1 in the attention and commit descriptors
 *     describes that: the tensors of the tree block (q, out, k_tree, v_tree) carry
 *     1 + N rows, row 0 = the root and row 1 + i = candidate i; every candidate
 *     attends to the prefix, the root, its ancestors and itself, the root to the prefix
 *     and itself; the commit appends the root and then the accepted path.  parent[]
 *     keeps its N entries and its meaning.  N + root_row <= MCSD_MAX_NODES.
 */
#ifndef MCSD_H
#define MCSD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MCSD_MAX_NODES 128      /* tree nodes per sequence (root excluded) */
#define MCSD_MAX_VOCAB 65536    /* the target row of a node stays in one workgroup's registers */
#define MCSD_MAX_HEAD_DIM 256

enum {
    MCSD_OK = 0,
    MCSD_E_NULL = -1,         /* a required pointer is NULL */
    MCSD_E_SHAPE = -2,        /* a size is non-positive / inconsistent / struct_size wrong */
    MCSD_E_UNSUPPORTED = -3,  /* valid request this build has no kernel for */
    MCSD_E_TREE = -4,         /* N > MCSD_MAX_NODES or parent[] not in parents-first order */
    MCSD_E_WORKSPACE = -5,    /* workspace missing, too small or misaligned (256 B) */
    MCSD_E_HIP = -6           /* the HIP runtime reported an error at launch */
};

enum { MCSD_DTYPE_FP32 = 0, MCSD_DTYPE_BF16 = 1 };
enum { MCSD_WITH_REPLACEMENT = 0, MCSD_WITHOUT_REPLACEMENT = 1,
       MCSD_NAIVE = 2 /* verification only: multi-candidate naive sampling, the ablation's comparison rule */ };

/* bits of mcsd_verify_bufs.flags[b][row] */
enum {
    MCSD_FLAG_NEAR_TIE_ACCEPT = 1,    /* an accept test had |u - ratio| < near_tie_eps */
    MCSD_FLAG_NEAR_TIE_ENDPOINT = 2,  /* u_endpoint within near_tie_eps of an edge of the chosen CDF interval */
    MCSD_FLAG_BAD_TOKEN = 4,          /* candidate id outside [0, V): treated as rejected */
    MCSD_FLAG_ZERO_DRAFT_PROB = 8,    /* q(candidate) == 0: ratio taken as 1 if p > 0 else 0 */
    MCSD_FLAG_ZERO_RESIDUAL = 16,     /* sum max(0, p - q) was not positive after a rejection */
    MCSD_FLAG_NONFINITE = 32,         /* a softmax normaliser was not finite and positive */
    MCSD_FLAG_BAD_TREE = 64,          /* a row with children has no valid q_row entry: handled as a leaf; or the walk
                                         reached gamma_max on a row that accepted a child (tree deeper than gamma_max) */
    MCSD_FLAG_NEAR_TIE_DRAW = 128,    /* mcsd_draft_sample: u_draw within near_tie_eps of an edge of the chosen CDF interval */
    MCSD_FLAG_CACHE_FULL = 256        /* mcsd_kv_commit: prefix_len + n_accepted > L_stride, nothing committed for this sequence */
};

const char *mcsd_last_error(void);
const char *mcsd_version(void);

/* Host-side check of a parent array (host pointer): MCSD_OK or MCSD_E_TREE / MCSD_E_NULL. */
int32_t mcsd_tree_validate(const int32_t *parent_host, int32_t n_nodes);

/* ------------------------------------------------------------- tree attention
 * Sec. 3.3.  For sequence b, query head h (KV head g = h / (H_q / H_kv)) and node i:
 *   keys   = prefix positions 0 .. prefix_len[b]-1  and  tree nodes in A(i),
 *            A(i) = {i} U A(parent[i]),  A(-1) = {}
 *   out[b][i][h][:] = softmax_over_keys(scale * <q[b][i][h], K>) . V
 * Inputs are expected to be position-encoded already (each candidate keeps the
 * position it has in its own sequence, i.e. prefix_len + depth - 1).
 * fp32 accumulation; bf16 inputs use the matrix cores when d == 128.
 */
typedef struct {
    uint32_t struct_size;
    int32_t B;              /* sequences */
    int32_t N;              /* tree nodes per sequence, 1..MCSD_MAX_NODES */
    int32_t H_q, H_kv;      /* query / KV heads, H_q % H_kv == 0 */
    int32_t d;              /* head dim: multiple of 4 (fp32) or 8 (bf16), <= MCSD_MAX_HEAD_DIM */
    int32_t dtype;          /* MCSD_DTYPE_* of q, k_*, v_*, out */
    int32_t L_stride;       /* rows allocated per (sequence, KV head) in the prefix cache; prefix_len[b] <= L_stride <= 2^22 */
    float scale;            /* softmax scale, finite and >= 0, normally 1/sqrt(d) */
    int32_t parent_per_seq; /* 0: one parent[N] shared by the batch; 1: parent[B][N] */
    int32_t root_row;       /* 0: the root is in the prefix cache; 1: the tree block has 1+N rows, row 0 = the root */
} mcsd_attn_desc;

typedef struct {
    uint32_t struct_size;
    const void *q;               /* [B][N][H_q][d]   (N here and below: N + root_row rows) */
    const void *k_prefix;        /* [B][H_kv][L_stride][d] */
    const void *v_prefix;        /* [B][H_kv][L_stride][d] */
    const int32_t *prefix_len;   /* [B], 0 <= prefix_len[b] <= L_stride */
    const void *k_tree;          /* [B][H_kv][N][d] */
    const void *v_tree;          /* [B][H_kv][N][d] */
    const int32_t *parent;       /* [N] or [B][N] */
    void *out;                   /* [B][N][H_q][d] */
    void *workspace;             /* >= mcsd_attn_workspace_bytes(desc), 256-byte aligned */
    size_t workspace_bytes;
} mcsd_attn_bufs;

/* Bytes of scratch mcsd_tree_attn needs for this descriptor (0 on a bad descriptor). */
size_t mcsd_attn_workspace_bytes(const mcsd_attn_desc *desc);
int32_t mcsd_tree_attn(const mcsd_attn_desc *desc, const mcsd_attn_bufs *bufs, void *stream);

/* The same operation for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The
 * split partials go to a buffer of MCSD_STATIC_SCRATCH_BYTES that is part of the library's
 * device image (one copy per GPU, held until the process ends) instead of bufs->workspace,
 * which is ignored together with bufs->workspace_bytes.  Inputs, outputs, stream semantics and
 * results (bit for bit) are those of mcsd_tree_attn.  The call allocates nothing and calls no
 * allocating routine.  A shape whose partials need more than MCSD_STATIC_SCRATCH_BYTES
 * (mcsd_attn_workspace_bytes tells) is refused with MCSD_E_WORKSPACE before anything is enqueued.
 * The first call on a device looks the buffer's address up (module set-up; make it outside
 * graph capture); `stream` must belong to the device that is current at the call.  All calls
 * on one GPU share the one buffer: calls that may overlap on a GPU (different streams, or
 * different host threads on unordered streams) race and must be ordered by the caller.
 * Nothing in the buffer has to survive from one call to the next. */
#define MCSD_STATIC_SCRATCH_BYTES ((size_t)96 << 20)
int32_t mcsd_tree_attn_static(const mcsd_attn_desc *desc, const mcsd_attn_bufs *bufs, void *stream);

/* Test and tuning aid, not needed in normal use: overrides the launch plan of the matrix-core
 * attention kernel for all later calls of this process (0 = automatic for each value).
 * variant 1, 2, 3 = the 32-row x 4-key-stream, 64-row x 2-key-stream and shared-tile kernels;
 * chunk_tiles = 32-key tiles per segment; target_items = workgroups aimed at when the segment
 * length is derived.  The workspace size depends on the plan: query mcsd_attn_workspace_bytes
 * after changing it.  MCSD_E_SHAPE for values out of range. */
int32_t mcsd_attn_plan_override(int32_t variant, int32_t chunk_tiles, int32_t target_items);

/* Paged prefix cache.  The same operation, but the prefix keys and values live in a pool of
 * fixed-size pages shared by all sequences (the usual serving layout): bufs->k_prefix and
 * bufs->v_prefix point to pools [n_pages][H_kv][page_size][d], and logical prefix row r of
 * sequence b is row r % page_size of page block_table[b][r / page_size].  page_size is a
 * multiple of 32; desc->L_stride is the logical capacity, <= max_pages_per_seq * page_size;
 * only the pages that hold rows below prefix_len[b] are read.  A table entry outside
 * [0, n_pages) is a data error: its keys read as zeros (bf16 matrix-core path) or as page 0 /
 * n_pages-1 (other paths); memory outside the pool is never touched.  Everything else (tree
 * block, outputs, workspace) is as for mcsd_tree_attn.
 */
typedef struct {
    uint32_t struct_size;
    int32_t page_size;              /* tokens per page, multiple of 32 */
    int32_t n_pages;                /* pages in the pools */
    int32_t max_pages_per_seq;      /* row length of block_table */
    const int32_t *block_table;     /* [B][max_pages_per_seq] device */
} mcsd_paged_kv;

int32_t mcsd_tree_attn_paged(const mcsd_attn_desc *desc, const mcsd_attn_bufs *bufs, const mcsd_paged_kv *paged,
                             void *stream);

/* --------------------------------------------------------------- verification
 * Algorithm 1 / Algorithm 2 for every row that has children, endpoint draws,
 * and the walk (Sec. 3).  Per sequence b with temperature T = temperature[b]:
 *   p_r = softmax(target_logits[b][r] / T),  q_r = softmax(draft_logits[b][q_row[r]] / T)
 *   for the children c_1 < c_2 < ... of row r, x = cand_tok[b][c_i]:
 *       ratio = min(1, p_r(x) / q_r(x));  accept c_i iff u_accept[b][c_i] <= ratio and ratio > 0
 *       else p_r := max(0, p_r - q_r) / sum_x max(0, p_r - q_r)
 *            and, without replacement only, q_r(x) := 0, q_r := q_r / sum q_r
 *   no child accepted, or r is a leaf: endpoint = inverse CDF of p_r (token-id
 *       order, smallest x whose cumulative probability exceeds u_endpoint[b][r])
 *   walk: r = 0; while a child c of r was accepted: emit cand_tok[c], r = 1 + c;
 *       then emit the endpoint of r.
 *   variant MCSD_NAIVE (Sec. 4.5, footnote; naive sampling of Sec. 2 for one candidate): a
 *       token x is drawn from p_r by inverse CDF at u_endpoint[b][r]; the first child whose
 *       token equals x is accepted, otherwise x is the endpoint; draft logits and u_accept
 *       are not read, ratio is NaN.
 *   T == 0 (argmax sampling, Sec. 4.1/4.5): accept the first child whose token is
 *       argmax target_logits[b][r] (lowest id on ties), otherwise that argmax is
 *       the endpoint; draft logits and uniforms are not read.
 * Every row is evaluated (not only the rows on the accepted path), so results do
 * not depend on evaluation order; uniforms are indexed by slot for the same reason.
 * Elementwise math in fp32 with fp64 reductions; the quantities that decide an
 * accept test are evaluated in fp64.
 */
typedef struct {
    uint32_t struct_size;
    int32_t B;
    int32_t N;              /* tree nodes per sequence, 1..MCSD_MAX_NODES */
    int32_t V;              /* vocabulary, 1..MCSD_MAX_VOCAB */
    int32_t P;              /* rows of draft_logits per sequence (rows of the tree that have children) */
    int32_t variant;        /* MCSD_WITH_REPLACEMENT | MCSD_WITHOUT_REPLACEMENT | MCSD_NAIVE */
    int32_t gamma_max;      /* depth bound: row length of accepted_path; out_tokens rows have gamma_max+1 */
    float near_tie_eps;     /* threshold of the MCSD_FLAG_NEAR_TIE_* bits, e.g. 1e-6 */
    int32_t parent_per_seq; /* 0: one tree for the batch (parent[N], q_row[1+N]); 1: one tree per
                               sequence (parent[B][N], q_row[B][1+N]): Sec. 3 verifies each sequence's
                               own candidate tree */
} mcsd_verify_desc;

typedef struct {
    uint32_t struct_size;
    const float *target_logits;  /* [B][1+N][V]   row 0 = root */
    const float *draft_logits;   /* [B][P][V] */
    const int32_t *q_row;        /* [1+N] or [B][1+N]: row of draft_logits for each tree row, -1 for leaves */
    const int32_t *parent;       /* [N] or [B][N] (desc->parent_per_seq) */
    const int32_t *cand_tok;     /* [B][N] candidate token of each node */
    const float *u_accept;       /* [B][N]   uniform in (0,1) for each node's accept test */
    const float *u_endpoint;     /* [B][1+N] uniform in (0,1) for each row's endpoint draw */
    const float *temperature;    /* [B], 0 = argmax sampling */
    int32_t *n_accepted;         /* [B] out: accepted candidates, 0..gamma_max */
    int32_t *accepted_path;      /* [B][gamma_max] out: node ids root-to-leaf, -1 padded */
    int32_t *out_tokens;         /* [B][gamma_max+1] out: accepted tokens then the endpoint, -1 padded */
    int32_t *acc_child;          /* [B][1+N] out: accepted child of each row or -1 */
    int32_t *endpoint;           /* [B][1+N] out: endpoint token of each row, -1 if a child was accepted */
    float *ratio;                /* [B][N] out, nullable: min(1, p/q) tested for each node, NaN if not reached */
    uint32_t *flags;             /* [B][1+N] out: MCSD_FLAG_* bits */
    float *residual_out;         /* [B][1+N][V] out, nullable (parity checks only): p_r when the loop ended */
    void *workspace;             /* unused by this build: may be NULL when mcsd_verify_workspace_bytes is 0 */
    size_t workspace_bytes;
} mcsd_verify_bufs;

size_t mcsd_verify_workspace_bytes(const mcsd_verify_desc *desc);
int32_t mcsd_verify_sample(const mcsd_verify_desc *desc, const mcsd_verify_bufs *bufs, void *stream);

/* One verification step: mcsd_tree_attn and mcsd_verify_sample on `stream`.  Both argument sets
 * are validated before anything is enqueued.  The results are those of the two calls made one
 * after the other; the launches may be arranged differently (the merge of a split attention
 * and the walk share one launch after the verification rows). */
int32_t mcsd_verify_step(const mcsd_attn_desc *attn_desc, const mcsd_attn_bufs *attn_bufs,
                         const mcsd_verify_desc *verify_desc, const mcsd_verify_bufs *verify_bufs,
                         void *stream);

/* ------------------------------------------------------- draft-side candidates
 * Sec. 3.1: the k candidates of every row that has children, sampled from the
 * draft distribution q_r = softmax(draft_logits[b][q_row[r]] / T); this is the
 * step just before verification and its output is the cand_tok input above.
 * For the children c_1 < c_2 < ... < c_k of row r:
 *   MCSD_WITH_REPLACEMENT     cand_tok[b][c_i] = inverse CDF of q_r at u_draw[b][c_i]
 *                             (token-id order, smallest x whose cumulative probability
 *                             exceeds the uniform): k independent draws, Algorithm 1's input;
 *   MCSD_WITHOUT_REPLACEMENT  the same, but draw i is taken from q_r with the tokens
 *                             of draws 1..i-1 zeroed and the rest renormalised (q-bar of
 *                             Eq. (1)): k distinct tokens, Algorithm 2's input;
 *   T == 0                    the k largest draft logits in descending order, lowest id
 *                             on ties; uniforms are not read.
 * Entries of cand_tok whose parent row has no valid q_row are set to -1 and flagged
 * MCSD_FLAG_BAD_TREE.  Requires k <= V for every row.  Elementwise math in fp32
 * (the same exponentials as mcsd_verify_sample), cumulative sums in fp64.
 */
typedef struct {
    uint32_t struct_size;
    int32_t B;
    int32_t N;              /* tree nodes per sequence, 1..MCSD_MAX_NODES */
    int32_t V;              /* vocabulary, 1..MCSD_MAX_VOCAB */
    int32_t P;              /* rows of draft_logits per sequence */
    int32_t variant;        /* MCSD_WITH_REPLACEMENT | MCSD_WITHOUT_REPLACEMENT */
    float near_tie_eps;     /* threshold of MCSD_FLAG_NEAR_TIE_DRAW, e.g. 1e-6 */
    int32_t parent_per_seq; /* 0: one tree for the batch; 1: parent[B][N], q_row[B][1+N] */
} mcsd_draft_desc;

typedef struct {
    uint32_t struct_size;
    const float *draft_logits;   /* [B][P][V], 16-byte aligned */
    const int32_t *q_row;        /* [1+N] or [B][1+N]: row of draft_logits for each tree row, -1 for leaves */
    const int32_t *parent;       /* [N] or [B][N] (desc->parent_per_seq) */
    const float *u_draw;         /* [B][N] uniform in (0,1) for each node's draw */
    const float *temperature;    /* [B], 0 = top-k */
    int32_t *cand_tok;           /* [B][N] out */
    uint32_t *flags;             /* [B][N] out: MCSD_FLAG_NEAR_TIE_DRAW / MCSD_FLAG_BAD_TREE / MCSD_FLAG_NONFINITE per node */
} mcsd_draft_bufs;

int32_t mcsd_draft_sample(const mcsd_draft_desc *desc, const mcsd_draft_bufs *bufs, void *stream);

/* ------------------------------------------------ candidate tree and KV commit
 * The two bookkeeping steps around the verification, on the device so that a
 * decode loop needs no host round trip (prefix_len lives in device memory).
 *
 * mcsd_tree_size / mcsd_tree_build: the k-ary candidate tree of a k-configuration
 * (k_1 .. k_gamma; Sec. 3 and Sec. 4.3), in the generation order in which Sec. 3.3
 * packs the candidates into one sequence: level by level, every node of level i-1
 * (the root for i = 1) gets k_i consecutive children.
 *   parent[N], depth[N] (1-based), q_row[1+N] (draft row of every tree row with
 *   children, numbered in row order; -1 for leaves),
 *   position_ids[B][N] = prefix_len[b] + depth[i] - 1 (each candidate keeps the
 *   position it has in its own sequence; nullable, then prefix_len may be NULL too);
 *   with root_row = 1, position_ids[B][1+N]: entry 0 = prefix_len[b] (the root, first
 *   token after the cache), entry 1 + i = prefix_len[b] + depth[i].
 * kconfig is HOST memory (gamma <= 16 entries, each >= 1); N must not exceed
 * MCSD_MAX_NODES (MCSD_E_TREE).  mcsd_tree_size only computes N and P on the host.
 */
int32_t mcsd_tree_size(const int32_t *kconfig_host, int32_t gamma, int32_t *n_nodes, int32_t *n_draft_rows);
int32_t mcsd_tree_build(const int32_t *kconfig_host, int32_t gamma, int32_t B, const int32_t *prefix_len,
                        int32_t *parent, int32_t *depth, int32_t *q_row, int32_t *position_ids, int32_t root_row,
                        void *stream);

/* mcsd_kv_commit: keys and values of generated tokens are cached for reuse (Sec. 3.3);
 * after verification the accepted candidates are generated tokens.  For sequence b with
 * n = n_accepted[b] and L = prefix_len[b], and every layer and KV head:
 *   k_prefix[layer][b][g][L + j] = k_tree[layer][b][g][accepted_path[b][j]],  j = 0..n-1 (same for V)
 *   prefix_len[b] = L + n;  next_root[b] = out_tokens[b][n]  (the endpoint, root of the next tree)
 * If L + n > L_stride nothing is copied, prefix_len[b] is left alone and flags[b] gets
 * MCSD_FLAG_CACHE_FULL (0 otherwise); path entries outside [0, N) end the copy there and set
 * MCSD_FLAG_BAD_TREE.  n_accepted, accepted_path and out_tokens are the outputs of
 * mcsd_verify_sample.  The caches of n_layers layers lie back to back.
 * With root_row = 1 (k_tree, v_tree have 1 + N rows, row 0 = the root, see the conventions):
 *   k_prefix[..][L] = k_tree[..][0],  k_prefix[..][L + 1 + j] = k_tree[..][1 + accepted_path[b][j]],
 *   prefix_len[b] = L + 1 + n;  the cache is full if L + 1 + n > L_stride.
 * The sequence held by the cache after the commit is then: context, root, accepted tokens; the
 * endpoint (next_root) is the root row of the next step.
 */
typedef struct {
    uint32_t struct_size;
    int32_t B;
    int32_t N;              /* tree nodes per sequence, 1..MCSD_MAX_NODES */
    int32_t H_kv;
    int32_t d;              /* head dim; d * element size must be a multiple of 16 bytes */
    int32_t dtype;          /* MCSD_DTYPE_* of the caches */
    int32_t L_stride;       /* rows allocated per (sequence, KV head) in the prefix cache */
    int32_t gamma_max;      /* row length of accepted_path; out_tokens rows have gamma_max+1 */
    int32_t n_layers;       /* >= 1 */
    int32_t root_row;       /* 0 | 1, as in mcsd_attn_desc */
} mcsd_commit_desc;

typedef struct {
    uint32_t struct_size;
    void *k_prefix;                 /* [n_layers][B][H_kv][L_stride][d] in/out */
    void *v_prefix;                 /* [n_layers][B][H_kv][L_stride][d] in/out */
    const void *k_tree;             /* [n_layers][B][H_kv][N + root_row][d] */
    const void *v_tree;             /* [n_layers][B][H_kv][N + root_row][d] */
    const int32_t *n_accepted;      /* [B] */
    const int32_t *accepted_path;   /* [B][gamma_max] */
    const int32_t *out_tokens;      /* [B][gamma_max+1] */
    int32_t *prefix_len;            /* [B] in/out */
    int32_t *next_root;             /* [B] out */
    uint32_t *flags;                /* [B] out */
} mcsd_commit_bufs;

int32_t mcsd_kv_commit(const mcsd_commit_desc *desc, const mcsd_commit_bufs *bufs, void *stream);

/* The same commit into a paged prefix cache (layout of mcsd_tree_attn_paged): bufs->k_prefix and
 * bufs->v_prefix are pools [n_layers][n_pages][H_kv][page_size][d], and row L + j of sequence b
 * is row (L + j) % page_size of page block_table[b][(L + j) / page_size]; the pages must already
 * be assigned in the table.  desc->L_stride is the logical capacity (<= max_pages_per_seq *
 * page_size).  A table entry outside [0, n_pages) ends the copy of that sequence there and sets
 * MCSD_FLAG_BAD_TREE; nothing outside the pools is written. */
int32_t mcsd_kv_commit_paged(const mcsd_commit_desc *desc, const mcsd_commit_bufs *bufs, const mcsd_paged_kv *paged,
                             void *stream);

/* ------------------------------------------------------------ profiling aid
 * Not part of the verification step.  mcsd_kernel_timing(1) makes every kernel launch of the
 * calls above carry a start and a stop event tied to that one dispatch (totals are reset), so
 * that the time between them is the kernel's own execution time, without launch latency or
 * the gaps between kernels; mcsd_kernel_timing(0) stops.  mcsd_kernel_timing_read waits for
 * the recorded events and returns the summed duration (ms) and the number of launches of
 * kernel `id` (0 .. mcsd_kernel_count()-1, named by mcsd_kernel_name).  Events are host
 * objects; no device memory is allocated.  Not for use under graph capture.
 */
int32_t mcsd_kernel_timing(int32_t enable);
int32_t mcsd_kernel_count(void);
const char *mcsd_kernel_name(int32_t id);
int32_t mcsd_kernel_timing_read(int32_t id, double *total_ms, int64_t *launches);

#ifdef __cplusplus
}
#endif
#endif /* MCSD_H */
