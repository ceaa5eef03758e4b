// Bookkeeping around the verification step, on the device: the candidate tree of a
// k-configuration (Sec. 3 / Sec. 4.3, generation order of Sec. 3.3) and the commit of the
// accepted path's keys and values to the prefix cache (Sec. 3.3).  Latency-sized kernels.
#include "mcsd_internal.h"

namespace mcsd {
namespace {

struct TreeParams {
    int k[MAX_GAMMA];
    int gamma, N, B, root_row;
    const int32_t *prefix_len;
    int32_t *parent, *depth, *q_row, *position_ids;
};

// One workgroup: thread i builds node i.  Level l (1-based) holds k_1 ... k_l nodes, its first
// node id is the sum of the earlier level sizes; node j of a level is child number j % k_l of
// node j / k_l of the level above.  Rows with children are exactly the rows above the last
// level, so their draft rows are numbered by the row index itself.
__global__ __launch_bounds__(256) void tree_build_kernel(TreeParams p)
{
    const int i = threadIdx.x;
    __shared__ int s_depth[MCSD_MAX_NODES];
    int internal_rows = 1;
    if (i < p.N) {
        int begin = 0, size = 1, prev_begin = -1, lvl = 0;
        for (int l = 1; l <= p.gamma; ++l) {
            const int sz = size * p.k[l - 1];
            if (i < begin + sz) {
                const int j = i - begin;
                p.parent[i] = (l == 1) ? -1 : prev_begin + j / p.k[l - 1];
                lvl = l;
                break;
            }
            prev_begin = begin;
            begin += sz;
            size = sz;
        }
        p.depth[i] = lvl;
        s_depth[i] = lvl;
    }
    {
        int size = 1;
        for (int l = 1; l < p.gamma; ++l) { size *= p.k[l - 1]; internal_rows += size; }
    }
    if (i <= p.N) p.q_row[i] = (i < internal_rows) ? i : -1;
    if (p.position_ids) {
        __syncthreads();
        // Without a root row the root is the last token of the prefix (position prefix_len - 1) and
        // a candidate of depth j sits at prefix_len + j - 1; with one, the root is the first new
        // token (entry 0, position prefix_len) and the candidates follow it.
        const int rows = p.N + p.root_row;
        for (int e = i; e < p.B * rows; e += blockDim.x) {
            const int b = e / rows, r = e % rows;
            p.position_ids[e] = p.root_row ? p.prefix_len[b] + (r == 0 ? 0 : s_depth[r - 1])
                                           : p.prefix_len[b] + s_depth[r] - 1;
        }
    }
}

struct CommitParams {
    int B, N, H_kv, L_stride, gamma_max, n_layers, root_row;
    int row_bytes;          // d * element size, multiple of 16
    char *k_prefix, *v_prefix;
    const char *k_tree, *v_tree;
    const int32_t *n_accepted, *accepted_path, *out_tokens;
    int32_t *prefix_len, *next_root;
    uint32_t *flags;
    // paged destination (block_table != nullptr): pools [n_layers][n_pages][H_kv][page_size][d]
    const int32_t *block_table;
    int page_size, n_pages, max_pages;
};

// Rows of a paged cache that can be committed for sequence b starting at logical row L: the
// first `n` rows whose pages are inside the pool.
__device__ __forceinline__ int paged_rows_ok(const CommitParams &p, int b, long L, int n)
{
    int good = 0;
    while (good < n) {
        const int blk = p.block_table[(size_t)b * p.max_pages + (L + good) / p.page_size];
        if ((unsigned)blk >= (unsigned)p.n_pages) break;
        ++good;
    }
    return good;
}

// grid (gamma_max + root_row, B, n_layers): block (j, b, layer) copies entry j of sequence b, all
// KV heads, K and V.  Without a root row, entry j is path entry j.  With one (the tree block has
// 1 + N rows, row 0 = the root, whose keys and values this forward pass produced as well), entry 0
// is the root and entry j >= 1 path entry j - 1: the root goes to cache row L, the candidate of
// depth j to row L + j.  prefix_len is only read here; kv_finish_kernel updates it afterwards.
__global__ __launch_bounds__(256) void kv_copy_kernel(CommitParams p)
{
    const int j = blockIdx.x, b = blockIdx.y, layer = blockIdx.z;
    const int n = p.n_accepted[b];
    if (n < 0 || n > p.gamma_max) return;
    const int n_rows = n + p.root_row;          // cache rows this sequence gains
    if (j >= n_rows) return;
    const long L = p.prefix_len[b];
    if (L < 0 || L + n_rows > p.L_stride) return;
    // a bad entry anywhere before j stops the copy there (the finish kernel reports it)
    for (int e = 0; e <= j - p.root_row; ++e) {
        const int nd = p.accepted_path[(size_t)b * p.gamma_max + e];
        if (nd < 0 || nd >= p.N) return;
    }
    const int tree_rows = p.N + p.root_row;
    const int src_row = (p.root_row && j == 0) ? 0 : p.root_row + p.accepted_path[(size_t)b * p.gamma_max + (j - p.root_row)];
    const int vec_per_row = p.row_bytes / 16;
    const size_t lb = (size_t)layer * p.B + b;
    size_t page_base = 0;       // paged: first row of the destination page slice of KV head 0
    if (p.block_table) {
        if (paged_rows_ok(p, b, L, j + 1) <= j) return;      // this row's page, or an earlier one, is not in the pool
        const int blk = p.block_table[(size_t)b * p.max_pages + (L + j) / p.page_size];
        page_base = ((size_t)layer * p.n_pages + blk) * (size_t)p.H_kv * p.page_size + (size_t)((L + j) % p.page_size);
    }
    for (int e = threadIdx.x; e < p.H_kv * vec_per_row; e += blockDim.x) {
        const int g = e / vec_per_row, c = e % vec_per_row;
        const size_t src = ((lb * p.H_kv + g) * (size_t)tree_rows + src_row) * p.row_bytes + (size_t)c * 16;
        const size_t dst = (p.block_table ? page_base + (size_t)g * p.page_size
                                          : (lb * p.H_kv + g) * (size_t)p.L_stride + (size_t)(L + j)) * p.row_bytes + (size_t)c * 16;
        *reinterpret_cast<uint4 *>(p.k_prefix + dst) = *reinterpret_cast<const uint4 *>(p.k_tree + src);
        *reinterpret_cast<uint4 *>(p.v_prefix + dst) = *reinterpret_cast<const uint4 *>(p.v_tree + src);
    }
}

__global__ void kv_finish_kernel(CommitParams p)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= p.B) return;
    int n = p.n_accepted[b];
    uint32_t fl = 0u;
    if (n < 0 || n > p.gamma_max) { n = 0; fl |= (uint32_t)MCSD_FLAG_BAD_TREE; }
    p.next_root[b] = p.out_tokens[(size_t)b * (p.gamma_max + 1) + n];
    const long L = p.prefix_len[b];
    if (L < 0 || L + n + p.root_row > p.L_stride) {
        fl |= (uint32_t)MCSD_FLAG_CACHE_FULL;
    } else {
        int good = 0;
        while (good < n) {
            const int nd = p.accepted_path[(size_t)b * p.gamma_max + good];
            if (nd < 0 || nd >= p.N) { fl |= (uint32_t)MCSD_FLAG_BAD_TREE; break; }
            ++good;
        }
        int rows = good + p.root_row;           // cache rows gained: the root (if it has a row), then the path
        if (p.block_table) {
            const int ok = paged_rows_ok(p, b, L, rows);
            if (ok < rows) { fl |= (uint32_t)MCSD_FLAG_BAD_TREE; rows = ok; }
        }
        p.prefix_len[b] = (int32_t)(L + rows);
    }
    p.flags[b] = fl;
}

}  // namespace

int32_t launch_tree_build(const int32_t *kconfig, int gamma, int n_nodes, int B, const int32_t *prefix_len,
                          int32_t *parent, int32_t *depth, int32_t *q_row, int32_t *position_ids, int root_row, hipStream_t stream)
{
    TreeParams p = {};
    for (int i = 0; i < gamma; ++i) p.k[i] = kconfig[i];
    p.gamma = gamma; p.N = n_nodes; p.B = B; p.root_row = root_row; p.prefix_len = prefix_len;
    p.parent = parent; p.depth = depth; p.q_row = q_row; p.position_ids = position_ids;
    launch_kernel(K_TREE_BUILD, tree_build_kernel, dim3(1), dim3(256), stream, p);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_error("tree_build launch failed: %s", hipGetErrorString(e)); return MCSD_E_HIP; }
    return MCSD_OK;
}

int32_t launch_kv_commit(const mcsd_commit_desc &d, const mcsd_commit_bufs &b, hipStream_t stream,
                         const mcsd_paged_kv *paged)
{
    CommitParams p;
    p.block_table = nullptr; p.page_size = p.n_pages = p.max_pages = 0;
    if (paged) {
        p.block_table = paged->block_table; p.page_size = paged->page_size;
        p.n_pages = paged->n_pages; p.max_pages = paged->max_pages_per_seq;
    }
    p.B = d.B; p.N = d.N; p.H_kv = d.H_kv; p.L_stride = d.L_stride; p.gamma_max = d.gamma_max; p.n_layers = d.n_layers;
    p.root_row = d.root_row ? 1 : 0;
    p.row_bytes = d.d * (d.dtype == MCSD_DTYPE_FP32 ? 4 : 2);
    p.k_prefix = static_cast<char *>(b.k_prefix); p.v_prefix = static_cast<char *>(b.v_prefix);
    p.k_tree = static_cast<const char *>(b.k_tree); p.v_tree = static_cast<const char *>(b.v_tree);
    p.n_accepted = b.n_accepted; p.accepted_path = b.accepted_path; p.out_tokens = b.out_tokens;
    p.prefix_len = b.prefix_len; p.next_root = b.next_root; p.flags = b.flags;
    launch_kernel(K_KV_COPY, kv_copy_kernel, dim3(d.gamma_max + p.root_row, d.B, d.n_layers), dim3(256), stream, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_error("kv_copy launch failed: %s", hipGetErrorString(e)); return MCSD_E_HIP; }
    launch_kernel(K_KV_FINISH, kv_finish_kernel, dim3((d.B + 63) / 64), dim3(64), stream, p);
    e = hipGetLastError();
    if (e != hipSuccess) { set_error("kv_finish launch failed: %s", hipGetErrorString(e)); return MCSD_E_HIP; }
    return MCSD_OK;
}

}  // namespace mcsd
