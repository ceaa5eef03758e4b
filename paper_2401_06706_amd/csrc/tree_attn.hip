// Tree attention (Sec. 3.3 of the paper) on gfx950.
//
// All candidate tokens of the draft tree are scored in one pass over the shared
// prefix KV cache: the cache is streamed from HBM once and every tree node (times
// the query heads that share a KV head) is a row of the same tile, which is the
// saving the paper attributes to tree attention.  A node additionally attends to
// its ancestors and itself among the tree's own keys; that mask is a 128-bit
// ancestor bitmask per node held in LDS.
//
// Work decomposition (bf16, d = 128: tree_attn_mfma_kernel)
//   keys of a sequence = ceil(L/32) prefix tiles followed by ceil(N/32) tree tiles
//   unit      = (sequence b, KV head g, tile of 32/64/128 query rows)
//   segment   = a run of consecutive key tiles of a unit, processed by one workgroup
//               (4 waves): wave (rh, ks) owns 32 rows and every KS-th tile of the run and
//               runs an independent online softmax with no workgroup barrier in the loop
//               (32- and 64-row tiles), or four waves of 32 rows walk one key stream together
//               and share every tile through LDS (128-row tiles, more than 64 rows per KV head).
//   The T tiles of a unit are cut into round(T / chunk_tiles) equal segments (at least one):
//   grid (KV head, segment x row tile, sequence).  The (sequence, segment) pairs are handed
//   out longest first.  A segment that covers its whole unit writes the output rows itself;
//   otherwise its (max, sum, O) partial goes to the workspace and tree_attn_combine_kernel
//   merges the partials of a unit by log-sum-exp.
//   The prefix cache is either one contiguous slab per (sequence, KV head) or a pool of
//   pages addressed through a block table (PAGED instantiation); the tiles are the same.
//
// Everything else (fp32 storage, other head dims) runs tree_attn_generic_kernel on
// the vector ALUs.
#include <math.h>

#include <atomic>
#include <type_traits>

#include "mcsd_internal.h"

namespace mcsd {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr float LOG2E_F = 1.44269504088896340736f;
constexpr float M_INIT = -1.0e30f;     // "no key seen yet" running max (finite so that differences stay finite)
constexpr float RESCALE_GAP = 8.0f;    // running max is only raised when a score exceeds it by 2^8
constexpr int KT = 32;                 // keys per tile

struct AttnParams {
    const void *q, *k_prefix, *v_prefix, *k_tree, *v_tree;
    const int32_t *prefix_len, *parent;
    void *out;
    float *part_m, *part_l, *part_o;
    int B, N, H_q, H_kv, G, d, L_stride, M;
    int n_row_tiles, chunk_tiles, n_chunks_max, tiles_tree, parent_per_seq, dtype;
    int root_row;         // 1: row 0 of the tree block is the root, N counts it
    int R;                // rows per (b, g) in the partial buffers
    int split_bias;       // see split_tiles
    float scale_log2;     // scale * log2(e)
    // paged prefix cache (block_table != nullptr): k_prefix / v_prefix are pools
    // [n_pages][H_kv][page_size][d]; logical row r of sequence b lives in page
    // block_table[b][r / page_size], slot r % page_size
    const int32_t *block_table;
    int page_size, n_pages, max_pages;
};


__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    bf16x2 v = {(__bf16)lo, (__bf16)hi};
    return __builtin_bit_cast(uint32_t, v);
}

// Raw buffer resource over [ptr, ptr + bytes): reads past the end return zero.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *ptr, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(ptr), 0, bytes, 0x00020000);
}

// max(a, b, c) as the one hardware instruction: fmaxf() on values the compiler knows nothing
// about (matrix-instruction results) costs an extra NaN-quieting v_max_f32 x, x per operand.
__device__ __forceinline__ float max3_raw(float a, float b, float c)
{
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// A vector instruction that reads the result of a matrix instruction has to keep a distance
// from it (seven wait states for v_mfma_f32_16x16x32_bf16) which the hardware does not enforce.
// The compiler keeps it for the instructions it selects itself, but not for the text of an asm
// statement: the four score accumulators pass through this statement before max3_raw reads
// them, so every matrix instruction that writes them has been issued before its wait states
// and every reader stands behind them.
__device__ __forceinline__ void settle_scores(f32x4 &a, f32x4 &b, f32x4 &c, f32x4 &d)
{
    asm volatile("s_nop 7\n\ts_nop 1" : "+v"(a), "+v"(b), "+v"(c), "+v"(d));
}

// the largest of the eight scores a lane holds for one row (two accumulators of four)
__device__ __forceinline__ float max_of_scores(const f32x4 &s0, const f32x4 &s1)
{
    const float m0 = max3_raw(s0[0], s0[1], s0[2]);
    const float m1 = max3_raw(s0[3], s1[0], s1[1]);
    return max3_raw(max3_raw(m0, m1, s1[2]), s1[3], s1[3]);
}

__device__ __forceinline__ float fast_exp2(float x)
{
    return __builtin_amdgcn_exp2f(x);      // v_exp_f32; results below the normal range flush to 0
}

__device__ __forceinline__ float bf16_bits_to_float(uint32_t bits16)
{
    return __uint_as_float(bits16 << 16);
}

// The T key tiles of a sequence are cut into n segments of seg tiles (the last one possibly
// shorter): n = (T + bias) / chunk_tiles, at least 1.  With bias = chunk_tiles / 2 that is
// T / chunk_tiles rounded to nearest, so a sequence a little longer than a multiple of
// chunk_tiles does not pay a partial for a sliver; seg < 1.5 chunk_tiles.
__device__ __forceinline__ void split_tiles(int T, int chunk_tiles, int bias, int *n, int *seg)
{
    const int nn = max(1, (T + bias) / chunk_tiles);
    *n = nn;
    *seg = (T + nn - 1) / nn;
}

// anc[i] = {i} U anc[parent[i]]: one 128-bit mask per node, built by walking up.  The parent
// array is copied to LDS with one coalesced load first, so that the walk (one dependent read
// per level) does not pay a global-memory latency per step.  With a root row the tree block has
// N rows of which row 0 is the root and row 1 + i candidate i: the root is every candidate's
// ancestor, and the caller's array (N - 1 entries, -1 = child of the root) is shifted by one.
// Contains a workgroup barrier; the caller adds the one that publishes the masks.
__device__ __forceinline__ void build_ancestor_masks(const int32_t *parent, int N, int root_row, uint32_t (*s_anc)[4], int *s_parent)
{
    for (int i = threadIdx.x; i < MCSD_MAX_NODES; i += blockDim.x) {
        int pa = -1;
        if (i < N) {
            if (!root_row) pa = parent[i];
            else if (i > 0) pa = max(parent[i - 1], -1) + 1;
        }
        s_parent[i] = pa;
    }
    __syncthreads();
    for (int i = threadIdx.x; i < MCSD_MAX_NODES; i += blockDim.x) {
        uint32_t m[4] = {0u, 0u, 0u, 0u};
        if (i < N) {
            int a = i;
            for (int step = 0; step < MCSD_MAX_NODES && a >= 0; ++step) {
                m[a >> 5] |= 1u << (a & 31);
                const int pa = s_parent[a];
                a = (pa < a) ? pa : -1;      // a malformed array can not loop or index out of range
            }
        }
        s_anc[i][0] = m[0]; s_anc[i][1] = m[1]; s_anc[i][2] = m[2]; s_anc[i][3] = m[3];
    }
}

// --------------------------------------------------------------------- MFMA path
// RH = row groups per workgroup, KS = key streams per workgroup.  Wave (rh, ks) owns query rows
// [32 rh, 32 (rh+1)) of the workgroup's row tile and the key tiles t_begin + ks, + KS, ... of the
// segment.  Waves of one key stream read the same K/V tiles (the second read is served by the
// L1/L2 caches).
//
// Data movement per 32-key tile and wave (8 KB of K, 8 KB of V, one 8.5 KB LDS area):
//   K  global -> registers with fully contiguous 1 KB loads (issued one tile ahead),
//      registers -> LDS in MFMA-operand order (16-byte granules, XOR-swizzled so that
//      both the stores and the operand loads are bank-conflict free), LDS -> operand.
//      Loading K straight into operand registers would make neighbouring lanes read
//      different cache lines, which stalls the address path of the vector memory unit.
//   V  global -> registers (a lane reads 8 key rows x 16 contiguous bytes, neighbouring
//      lanes neighbouring bytes; one tile ahead), in-lane 8x8 transpose of the 16-bit
//      elements, registers -> the same LDS area -> operand (exchange inside 16-lane groups).
//
// COOP (one key stream, several row groups): the waves of the workgroup share every K/V tile.
// Each wave loads a quarter of the tile and stores it to a double-buffered LDS tile that all
// waves read their operands from after one workgroup barrier per tile; K in the operand order
// above, V in its natural order (row pitch 288 bytes) and read with the transposing LDS load,
// which hands a lane the four keys of one d column that the PV operand needs.  Per wave and
// tile that is a quarter of the global loads and LDS stores of the private scheme and no
// in-register transpose, which matters where the matrix cores are the limit (many query rows
// per KV head).
template <int RH, int KS, bool PAGED, bool COOP = false>
__global__ __launch_bounds__(RH * KS * 64) __attribute__((amdgpu_waves_per_eu(2, 2)))
void tree_attn_mfma_kernel(AttnParams p, WalkParams w)
{
    static_assert(!COOP || (KS == 1 && RH == 4), "the shared-tile scheme splits a tile over four waves of one key stream");
    // Rows of workgroups appended to the grid along y carry the walk of a verification that ran
    // before this launch on the same stream (one thread per sequence), when the caller asked for
    // that: a step whose attention needs no merge launch then has no launch for the walk either.
    if ((int)blockIdx.y >= p.n_chunks_max * p.n_row_tiles) {
        if (blockIdx.x == 0 && blockIdx.z == 0) {
            const int wb = ((int)blockIdx.y - p.n_chunks_max * p.n_row_tiles) * (RH * KS * 64) + (int)threadIdx.x;
            if (wb < w.B) walk_sequence(w, wb);
        }
        return;
    }
    constexpr int MT = 2;                   // 16-row MFMA tiles per wave
    constexpr int NW = RH * KS;
    constexpr int NT = NW * 64;
    constexpr int WROWS = 16 * MT;          // rows per wave
    constexpr int ROWS = WROWS * RH;        // rows per workgroup
    constexpr int D = 128;
    constexpr int TILE_BYTES = KT * D * 2;  // 8192
    constexpr int AREA_WORDS = WROWS * 68;  // per-wave LDS area: >= 2048 words of staging, WROWS x 68 floats in the epilogue
    static_assert(AREA_WORDS >= 2048, "staging needs 8 KB per wave");
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keeps tile indices and pointers scalar
    const int rh = wave / KS, ks = wave % KS;
    const int lj = lane >> 4, lc = lane & 15;

    __shared__ __attribute__((aligned(16))) uint32_t s_big[NW * AREA_WORDS];
    __shared__ uint32_t s_anc[MCSD_MAX_NODES][4];
    __shared__ int s_parent[MCSD_MAX_NODES];
    __shared__ float s_m[KS][ROWS], s_l[KS][ROWS];
    __shared__ float s_mstar[ROWS], s_linv[ROWS];
    __shared__ int s_pair_len[NT], s_pair_of_rank[NT], s_seq_L[NT];

    // LDS positions (in 16-byte granules inside this wave's area).
    //   K granule (row r, granule c) is the operand of lane (c & 3, r & 15) for (sub = r >> 4, kk = c >> 2):
    //   position (sub 4 + kk) 64 + (c & 3) 16 + ((r & 15) ^ c)
    uint32_t *area = s_big + wave * AREA_WORDS;
    uint32_t kst_pos[4];        // store position of K load i: kst_pos[i & 3] + (i >> 2) * 256
#pragma unroll
    for (int j = 0; j < 4; ++j) kst_pos[j] = (lc >> 2) * 64 + (lc & 3) * 16 + ((4 * j + lj) ^ lc);
    uint32_t kld_pos[4];        // operand position for kk: kld_pos[kk] + sub * 256
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) kld_pos[kk] = kk * 64 + lj * 16 + (lc ^ (4 * kk + lj));
    //   V: column 8 lc + e of the lane's 8x8 block is the operand of lane 8 (lc & 1) + e for d-tile
    //   lc >> 1.  Position of (d-tile nt, lane hi 8 + lo) in the k-group's 128 granules:
    //   nt 16 + hi 8 + (lo ^ ((2 nt + hi) & 7)): eight neighbouring lanes cover all banks in the
    //   stores (fixed e: 2 nt + hi = lc runs through eight values) and in the loads (fixed nt: lo does).
    const uint32_t vst_base = lj * 128 + lc * 8;            // store position = vst_base + (e ^ vst_x)
    const uint32_t vst_x = lc & 7;
    const uint32_t vld_base = lj * 128 + (lc >> 3) * 8;     // load position = vld_base + nt 16 + (vld_x ^ ((2 nt) & 7))
    const uint32_t vld_x = (lc & 7) ^ (lc >> 3);
    // Per-lane byte offsets inside a tile (row pitch 256 B).
    //   K load i (0..7): row 4 i + lj, 16-byte granule lc  ->  i * 1024 + lane * 16
    //   V load s (0..7): row (s < 4 ? 0 : 16) + 4 lj + (s & 3), granule lc
    const uint32_t k_lane_off = lane * 16;
    const uint32_t v_lane_off = lj * 1024 + lc * 16;
    // COOP: wave w loads K rows and V rows 8 w .. 8 w + 7 (load j = 0, 1: row 8 w + 4 j + lj, granule lc).
    //   A buffer is 2048 words of K (operand order) followed by 32 V rows of 72 words.
    constexpr int COOP_BUF_WORDS = 2048 + KT * 72;
    static_assert(!COOP || 2 * COOP_BUF_WORDS <= NW * AREA_WORDS, "the two tile buffers live in the epilogue areas");
    uint32_t coop_kst[2], coop_vst[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int i = 2 * wave + j;                 // K load index of the private scheme
        coop_kst[j] = 4 * ((lc >> 2) * 64 + (lc & 3) * 16 + ((4 * (i & 3) + lj) ^ lc) + (i >> 2) * 256);
        coop_vst[j] = 2048 + (4 * i + lj) * 72 + lc * 4;
    }
    //   transposing read for (sub, nt): the 16 lanes of a group point at keys 16 sub + 4 lj + (lc >> 2),
    //   d columns 16 nt + 4 (lc & 3) .. + 3; lane lc receives column 16 nt + lc of keys 16 sub + 4 lj + 0..3
    const uint32_t coop_vld = 2048 + (4 * lj + (lc >> 2)) * 72 + (lc & 3) * 2;     // + sub 16 x 72 + nt 8 words
    const float c2 = p.scale_log2;      // >= 0 (checked by the host)
    const uint16_t *qb = static_cast<const uint16_t *>(p.q);

    // ---- this workgroup's segment: unit (b, g, rt), tiles [t_begin, t_end) of total_tiles
    int b, g, rt, t_begin, t_end, total_tiles, L;
    bool direct;
    size_t part_row;                    // first row of this segment's partial in the workspace
    {
        // Workgroups start in the order z, y, x.  The (sequence, chunk) pairs are handed out
        // longest first (the short last chunks of the sequences fill the end of the launch
        // instead of a mostly idle last wave of workgroups): pair number r in dispatch order
        // takes the pair of rank r by length.  Done when the pairs fit one workgroup's threads.
        g = blockIdx.x; b = blockIdx.z;
        rt = blockIdx.y % p.n_row_tiles;
        int chunk = blockIdx.y / p.n_row_tiles;
        const int n_pairs = p.B * p.n_chunks_max;
        if (n_pairs <= NT && p.n_chunks_max > 1) {
            int my_len = 0;
            if (tid < n_pairs) {
                int Lb = p.prefix_len[tid / p.n_chunks_max];
                Lb = max(0, min(Lb, p.L_stride));
                const int Tb = (Lb + KT - 1) / KT + p.tiles_tree;
                int nb, segb;
                split_tiles(Tb, p.chunk_tiles, p.split_bias, &nb, &segb);
                my_len = max(0, min(segb, Tb - (tid % p.n_chunks_max) * segb));
                s_pair_len[tid] = my_len;
                if (tid % p.n_chunks_max == 0) s_seq_L[tid / p.n_chunks_max] = Lb;
            }
            __syncthreads();
            if (tid < n_pairs) {
                int rank = 0;
                for (int j = 0; j < n_pairs; ++j) {
                    const int lj2 = s_pair_len[j];
                    rank += (lj2 > my_len || (lj2 == my_len && j < tid)) ? 1 : 0;
                }
                s_pair_of_rank[rank] = tid;
            }
            __syncthreads();
            const int pair = s_pair_of_rank[blockIdx.z * p.n_chunks_max + chunk];
            b = __builtin_amdgcn_readfirstlane(pair / p.n_chunks_max);       // read from LDS: make it scalar again
            chunk = __builtin_amdgcn_readfirstlane(pair % p.n_chunks_max);
            L = __builtin_amdgcn_readfirstlane(s_seq_L[b]);      // already loaded and clamped: no second trip to memory
        } else {
            L = p.prefix_len[b];
            L = max(0, min(L, p.L_stride));
        }
        total_tiles = (L + KT - 1) / KT + p.tiles_tree;
        int n_seg, seg;
        split_tiles(total_tiles, p.chunk_tiles, p.split_bias, &n_seg, &seg);
        t_begin = chunk * seg;
        if (t_begin >= total_tiles) return;
        t_end = min(total_tiles, t_begin + seg);
        direct = (n_seg == 1);
        part_row = (((size_t)b * p.H_kv + g) * p.n_chunks_max + chunk) * (size_t)p.R + (size_t)rt * ROWS;
    }
    {
        const int tilesP = (L + KT - 1) / KT;
        const int row0 = rt * ROWS;

        // Q operand, held in registers: lane (lj, lc) has Q[row0 + WROWS rh + 16 mt + lc][32 kk + 8 lj .. +7]
        bf16x8 qreg[MT][4];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const int r = row0 + WROWS * rh + 16 * mt + lc;
            const bool ok = r < p.M;
            const int rr = ok ? r : p.M - 1;
            const int node = rr / p.G, hh = rr % p.G;
            const uint16_t *src = qb + (((size_t)b * p.N + node) * p.H_q + (size_t)g * p.G + hh) * D + 8 * lj;
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                u32x4 v = *reinterpret_cast<const u32x4 *>(src + 32 * kk);
                if (!ok) v = (u32x4){0u, 0u, 0u, 0u};
                qreg[mt][kk] = __builtin_bit_cast(bf16x8, v);
            }
        }

        f32x4 oacc[8][MT];
#pragma unroll
        for (int nt = 0; nt < 8; ++nt)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) oacc[nt][mt] = (f32x4){0.f, 0.f, 0.f, 0.f};
        float m_used[MT], l_part[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) { m_used[mt] = M_INIT; l_part[mt] = 0.f; }

        const size_t kv_head = (size_t)b * p.H_kv + g;
        // K and V of this (sequence, KV head) are read through buffer resources whose extent is
        // exactly the valid rows (prefix_len rows of the cache slab, N rows of the tree block):
        // the tile base is a scalar offset, the lane offset a constant, and rows past the end of
        // a partial tile read as zero instead of leaving the array (their scores are masked).
        // (paged cache: the prefix resources are empty and every prefix tile gets a resource of
        // its own over the page slice it lies in)
        const __amdgpu_buffer_rsrc_t rs_kpre = make_rsrc(static_cast<const char *>(p.k_prefix) + (PAGED ? 0 : kv_head * (size_t)p.L_stride * (D * 2)), PAGED ? 0u : (uint32_t)L * (D * 2));
        const __amdgpu_buffer_rsrc_t rs_vpre = make_rsrc(static_cast<const char *>(p.v_prefix) + (PAGED ? 0 : kv_head * (size_t)p.L_stride * (D * 2)), PAGED ? 0u : (uint32_t)L * (D * 2));
        const __amdgpu_buffer_rsrc_t rs_ktre = make_rsrc(static_cast<const char *>(p.k_tree) + kv_head * (size_t)p.N * (D * 2), (uint32_t)p.N * (D * 2));
        const __amdgpu_buffer_rsrc_t rs_vtre = make_rsrc(static_cast<const char *>(p.v_tree) + kv_head * (size_t)p.N * (D * 2), (uint32_t)p.N * (D * 2));

        struct TileRef { int off; int nvalid; bool tree; int tt; size_t page_off; bool paged; };
        // Tiles at or past t_end are requested at an offset beyond every buffer's extent: the
        // hardware returns zeros without touching memory.  This keeps the prefetch of the next
        // tile unconditional, so the wait for one tile's data never has to cover the loads issued
        // after it (a load under a branch makes the compiler wait for everything outstanding).
        constexpr int OFF_NOWHERE = 0x7fff0000;
        // (paged cache: blk = the block-table entry of the page the tile starts in)
        auto tile_ref_blk = [&](int t, int blk, int row_in_page) {
            TileRef r;
            r.page_off = 0; r.paged = false;
            if (t >= t_end) {
                r.off = OFF_NOWHERE; r.nvalid = KT; r.tree = false; r.tt = 0;
            } else if (t < tilesP) {
                r.off = t * TILE_BYTES; r.nvalid = min(KT, L - t * KT); r.tree = false; r.tt = 0;
                if (PAGED) {
                    if ((unsigned)blk < (unsigned)p.n_pages) {
                        r.paged = true;
                        r.off = 0;
                        r.page_off = (((size_t)blk * p.H_kv + g) * (size_t)p.page_size + (size_t)row_in_page) * (D * 2);
                    } else {
                        r.off = OFF_NOWHERE;       // an entry outside the pool reads as zero keys, never as memory
                    }
                }
            } else {
                r.tt = t - tilesP;
                r.off = r.tt * TILE_BYTES; r.nvalid = min(KT, p.N - r.tt * KT); r.tree = true;
            }
            return r;
        };
        // The block table is only read by this kernel.  Through a pointer to the constant address
        // space its (wave-uniform) entries are fetched with scalar loads wherever the read stands;
        // through the plain pointer the compiler falls back to a vector load behind every barrier
        // or asm statement, and the wait for that load covers all K/V requests in flight.
        typedef const int32_t __attribute__((address_space(4))) *const_i32_ptr;
        const const_i32_ptr block_table_c = (const_i32_ptr)(uintptr_t)p.block_table;
        auto tile_ref = [&](int t) {
            int blk = -1;
            if (PAGED && t < t_end && t < tilesP) blk = block_table_c[(size_t)b * p.max_pages + (t * KT) / p.page_size];
            return tile_ref_blk(t, blk, PAGED ? (t * KT) % p.page_size : 0);
        };
        u32x4 kraw[8];
        auto load_k = [&](const TileRef &r) {
            __amdgpu_buffer_rsrc_t rs = r.tree ? rs_ktre : rs_kpre;
            if (PAGED && r.paged) rs = make_rsrc(static_cast<const char *>(p.k_prefix) + r.page_off, (uint32_t)r.nvalid * (D * 2));
#pragma unroll
            for (int i = 0; i < 8; ++i) kraw[i] = __builtin_amdgcn_raw_buffer_load_b128(rs, k_lane_off + i * 1024, r.off, 0);
        };
        u32x4 vcur[8];
        auto load_v = [&](const TileRef &r) {
            __amdgpu_buffer_rsrc_t rs = r.tree ? rs_vtre : rs_vpre;
            if (PAGED && r.paged) rs = make_rsrc(static_cast<const char *>(p.v_prefix) + r.page_off, (uint32_t)r.nvalid * (D * 2));
#pragma unroll
            for (int s = 0; s < 8; ++s)
                vcur[s] = __builtin_amdgcn_raw_buffer_load_b128(rs, v_lane_off + ((s < 4) ? 0 : 4096) + (s & 3) * 256, r.off, 0);
        };

        // Paged cache, COOP: the block-table entry of a tile is read one step before the tile is
        // requested, ahead of the workgroup barrier.  Scalar loads share the LDS counter and
        // return out of order, so using one right after issuing it would drain every LDS read in
        // flight; at the barrier that wait is made anyway.  The page and the row inside it of the
        // tile that is looked up next advance by one tile per step (no division in the loop).
        int ahead_page = 0, ahead_row = 0;          // of the tile whose entry is read next
        int blk_ahead = -1, row_ahead = 0;          // entry and row-in-page read last
        auto table_lookup_next = [&](int tt) {      // tt = index of that tile
            row_ahead = ahead_row;
            blk_ahead = (PAGED && tt < tilesP && tt < t_end) ? (int)block_table_c[(size_t)b * p.max_pages + ahead_page] : -1;
            ahead_row += KT;
            if (ahead_row >= p.page_size) { ahead_row = 0; ++ahead_page; }
        };
        // COOP: this wave's quarter of both tiles (two K and two V requests)
        auto load_kv_coop = [&](const TileRef &r, const int st) {
            __amdgpu_buffer_rsrc_t rk = r.tree ? rs_ktre : rs_kpre;
            __amdgpu_buffer_rsrc_t rv = r.tree ? rs_vtre : rs_vpre;
            if (PAGED && r.paged) {
                rk = make_rsrc(static_cast<const char *>(p.k_prefix) + r.page_off, (uint32_t)r.nvalid * (D * 2));
                rv = make_rsrc(static_cast<const char *>(p.v_prefix) + r.page_off, (uint32_t)r.nvalid * (D * 2));
            }
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                kraw[2 * st + j] = __builtin_amdgcn_raw_buffer_load_b128(rk, k_lane_off + (2 * wave + j) * 1024, r.off, 0);
                vcur[2 * st + j] = __builtin_amdgcn_raw_buffer_load_b128(rv, k_lane_off + (2 * wave + j) * 1024, r.off, 0);
            }
        };

        int t = t_begin + ks;
        // (read before the first K/V requests, as inside the loop: the wait at the loop top is the
        // longer of the two paths into it)
        if (COOP && PAGED) {
            ahead_page = ((t + 3) * KT) / p.page_size;
            ahead_row = ((t + 3) * KT) % p.page_size;
            table_lookup_next(t + 3);
        }
        if (COOP) {
            // the first tile goes to its LDS buffer here, every later one inside the step before it;
            // requests run two to three tiles ahead of their use
            load_kv_coop(tile_ref(t), 0);
            load_kv_coop(tile_ref(t + 1), 1);
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                *reinterpret_cast<u32x4 *>(s_big + coop_kst[j]) = kraw[j];
                *reinterpret_cast<u32x4 *>(s_big + coop_vst[j]) = vcur[j];
            }
            load_kv_coop(tile_ref(t + 2), 0);
        } else {
            load_k(tile_ref(t));
            load_v(tile_ref(t));
        }
        const bool wave_active = !COOP || row0 + WROWS * rh < p.M;     // a wave whose rows all lie past M only helps to load
        // the masks are needed from the first tree tile on; built while the first loads are in flight
        if (t_end > tilesP) {
            build_ancestor_masks(p.parent + (p.parent_per_seq ? (size_t)b * (p.N - p.root_row) : 0), p.N, p.root_row, s_anc, s_parent);
            __syncthreads();
        }
        // PLAIN (a promise of the caller): tile t and the tile requested during this step are whole
        // prefix tiles inside the segment.  Nothing is masked, the step is one straight run of
        // instructions up to the (rare) raise of the running maxima, and with a contiguous cache
        // the tile references are plain offsets (a paged cache still looks its pages up).
        auto plain_ref = [&](int t) {
            TileRef r;
            r.off = t * TILE_BYTES; r.nvalid = KT; r.tree = false; r.tt = 0; r.page_off = 0; r.paged = false;
            return r;
        };
        auto tile_step = [&](const int t, auto stage, auto plain) __attribute__((always_inline)) {
            constexpr int ST = decltype(stage)::value;      // COOP: register stage and LDS buffer of this tile
            constexpr bool PLAIN = decltype(plain)::value;
            const TileRef cur = PLAIN ? plain_ref(t) : tile_ref(t);
            // Both K and V run one tile ahead of their use: K(t) goes from its load registers to LDS
            // (operand order) and K(t + KS) is requested into the same registers; V(t + KS) is
            // requested further down, as soon as V(t) has left its registers.
            if (COOP) {
                // Tile t is in buffer t & 1 once every wave has passed this barrier; tile t + 1 goes
                // from its registers to the other buffer while the matrix cores work on QK, and
                // tile t + 3 is requested into the registers that frees.  The other buffer is free:
                // it held tile t - 1, whose last read precedes every wave's arrival here.  One
                // barrier per tile, and no wave waits for memory or for its LDS stores at it.
                const uint32_t *cb = s_big + ST * COOP_BUF_WORDS;
                uint32_t *nb = s_big + (ST ^ 1) * COOP_BUF_WORDS;
                const int blk_next = blk_ahead, row_next = row_ahead;
                if (PAGED) table_lookup_next(t + 4);
                __syncthreads();
                typedef short v4i16 __attribute__((ext_vector_type(4)));
                typedef v4i16 __attribute__((address_space(3))) *lds_v4i16_ptr;
                f32x4 sacc[2][MT];
                if (wave_active) {
                    bf16x8 kop[4][2];
#pragma unroll
                    for (int kk = 0; kk < 4; ++kk) {
                        kop[kk][0] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(cb + 4 * kld_pos[kk]));
                        kop[kk][1] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(cb + 4 * (kld_pos[kk] + 256)));
                    }
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        sacc[0][mt] = (f32x4){0.f, 0.f, 0.f, 0.f};
                        sacc[1][mt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                        for (int kk = 0; kk < 4; ++kk) {
                            sacc[0][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kop[kk][0], qreg[mt][kk], sacc[0][mt], 0, 0, 0);
                            sacc[1][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kop[kk][1], qreg[mt][kk], sacc[1][mt], 0, 0, 0);
                        }
                    }
                }
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    *reinterpret_cast<u32x4 *>(nb + coop_kst[j]) = kraw[2 * (ST ^ 1) + j];
                    *reinterpret_cast<u32x4 *>(nb + coop_vst[j]) = vcur[2 * (ST ^ 1) + j];
                }
                load_kv_coop(PLAIN && !PAGED ? plain_ref(t + 3) : tile_ref_blk(t + 3, blk_next, row_next), ST ^ 1);
                if (!wave_active) return;
                // V^T operands by transposing LDS reads, requested now: they arrive during the first softmax
                bf16x8 vop[8];
#pragma unroll
                for (int nt = 0; nt < 8; ++nt) {
                    const v4i16 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16_ptr)(cb + coop_vld + nt * 8));
                    const v4i16 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16_ptr)(cb + coop_vld + 16 * 72 + nt * 8));
                    vop[nt] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
                }
                const bool masked = !PLAIN && (cur.nvalid < KT || cur.tree);
                uint32_t vis[MT];
                float lmax[MT];
                bool raise = false;
                settle_scores(sacc[0][0], sacc[0][1], sacc[1][0], sacc[1][1]);
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    vis[mt] = 0xffffffffu;
                    if (masked) {
                        const int node_m = min(row0 + WROWS * rh + 16 * mt + lc, p.M - 1) / p.G;
                        if (cur.tree) vis[mt] = s_anc[node_m][cur.tt];
                        if (cur.nvalid < KT) vis[mt] &= (1u << cur.nvalid) - 1u;
#pragma unroll
                        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                            for (int i = 0; i < 4; ++i)
                                if (!((vis[mt] >> (16 * sub + 4 * lj + i)) & 1u)) sacc[sub][mt][i] = -INFINITY;
                    }
                    // online softmax with a lazily raised running max (scaled, base-2 domain)
                    const float mr = max_of_scores(sacc[0][mt], sacc[1][mt]);
                    lmax[mt] = (mr == -INFINITY) ? -INFINITY : mr * c2;
                    raise |= lmax[mt] > m_used[mt] + RESCALE_GAP;
                }
                // one test for both row tiles: everything from here to the end of the step is one
                // straight run, in which the scheduler can place the vector work of one row tile
                // between the matrix instructions of the other
                if (__any(raise)) {
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        float rm = lmax[mt];
                        rm = fmaxf(rm, __shfl_xor(rm, 16));
                        rm = fmaxf(rm, __shfl_xor(rm, 32));
                        const float m_new = fmaxf(m_used[mt], rm);
                        const float alpha = fast_exp2(m_used[mt] - m_new);
                        m_used[mt] = m_new;
                        l_part[mt] *= alpha;
#pragma unroll
                        for (int nt = 0; nt < 8; ++nt) oacc[nt][mt] *= alpha;
                    }
                }
                // weights of one row tile: p = 2^(s c2 - m), masked keys 0; returns the lane's share of the row sum
                auto weights = [&](const int mt, bf16x8 &pop) __attribute__((always_inline)) {
                    float pv[8];
#pragma unroll
                    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                        for (int i = 0; i < 4; ++i) pv[4 * sub + i] = fast_exp2(fmaf(sacc[sub][mt][i], c2, -m_used[mt]));
                    if (masked) {
                        // also covers scale == 0, where a masked score can not be told apart by its value
#pragma unroll
                        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                            for (int i = 0; i < 4; ++i)
                                if (!((vis[mt] >> (16 * sub + 4 * lj + i)) & 1u)) pv[4 * sub + i] = 0.f;
                    }
                    const u32x4 pk = {pack_bf16(pv[0], pv[1]), pack_bf16(pv[2], pv[3]), pack_bf16(pv[4], pv[5]), pack_bf16(pv[6], pv[7])};
                    pop = __builtin_bit_cast(bf16x8, pk);
                    return ((pv[0] + pv[1]) + (pv[2] + pv[3])) + ((pv[4] + pv[5]) + (pv[6] + pv[7]));
                };
                // A wave issues in order, and vector instructions placed behind a matrix instruction
                // run while the matrix pipe works on it.  So: the weights of the first row tile; then
                // its eight PV matrix instructions, each followed by a share of the second row tile's
                // weights; then the second row tile's PV.  (O^T[d][row] += sum_key V[key][d] P[row][key])
                static_assert(MT == 2, "the schedule below is written for two row tiles per wave");
                bf16x8 pop0, pop1;
                const float sum0 = weights(0, pop0);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int nt = 0; nt < 8; ++nt)
                    oacc[nt][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vop[nt], pop0, oacc[nt][0], 0, 0, 0);
                const float sum1 = weights(1, pop1);
                l_part[0] += sum0;
                if (!masked) {
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                        __builtin_amdgcn_sched_group_barrier(0x402, 4, 0);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int nt = 0; nt < 8; ++nt)
                    oacc[nt][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vop[nt], pop1, oacc[nt][1], 0, 0, 0);
                l_part[1] += sum1;
                return;
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    *reinterpret_cast<u32x4 *>(area + 4 * (kst_pos[i & 3] + (i >> 2) * 256)) = kraw[i];
                load_k(PLAIN && !PAGED ? plain_ref(t + KS) : tile_ref(t + KS));
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            }

            // S^T[key][row] = sum_d K[key][d] Q[row][d]   (raw, the softmax scale is applied in the exponent)
            f32x4 sacc[2][MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) { sacc[0][mt] = (f32x4){0.f, 0.f, 0.f, 0.f}; sacc[1][mt] = (f32x4){0.f, 0.f, 0.f, 0.f}; }
            // operands are fetched from LDS four at a time ahead of the eight MFMAs that use them, so
            // that one LDS latency is exposed per group instead of one per operand
#pragma unroll
            for (int kh = 0; kh < 2; ++kh) {
                bf16x8 kop[2][2];
#pragma unroll
                for (int k2 = 0; k2 < 2; ++k2) {
                    const int kk = 2 * kh + k2;
                    kop[k2][0] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(area + 4 * kld_pos[kk]));
                    kop[k2][1] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(area + 4 * (kld_pos[kk] + 256)));
                }
#pragma unroll
                for (int k2 = 0; k2 < 2; ++k2)
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        sacc[0][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kop[k2][0], qreg[mt][2 * kh + k2], sacc[0][mt], 0, 0, 0);
                        sacc[1][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kop[k2][1], qreg[mt][2 * kh + k2], sacc[1][mt], 0, 0, 0);
                    }
            }
            // lane (lj, lc) now holds, for its row 16 mt + lc, keys 16 sub + 4 lj + i
            const bool masked = !PLAIN && (cur.nvalid < KT || cur.tree);
            uint32_t onmask[MT];
            if (masked) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    // the node of this lane's row is recomputed here (tree tiles are rare) rather than
                    // kept in a register across the whole loop
                    const int node_m = min(row0 + WROWS * rh + 16 * mt + lc, p.M - 1) / p.G;
                    uint32_t vis = cur.tree ? s_anc[node_m][cur.tt] : 0xffffffffu;
                    if (cur.nvalid < KT) vis &= (1u << cur.nvalid) - 1u;
                    onmask[mt] = vis;
#pragma unroll
                    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            if (!((vis >> (16 * sub + 4 * lj + i)) & 1u)) sacc[sub][mt][i] = -INFINITY;
                }
            }
            // online softmax with a lazily raised running max (scaled, base-2 domain)
            settle_scores(sacc[0][0], sacc[0][1], sacc[1][0], sacc[1][1]);
            bool raise = false;
            float lmax[MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const float mr = max_of_scores(sacc[0][mt], sacc[1][mt]);
                lmax[mt] = (mr == -INFINITY) ? -INFINITY : mr * c2;
                raise |= lmax[mt] > m_used[mt] + RESCALE_GAP;
            }
            if (__any(raise)) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    float rm = lmax[mt];
                    rm = fmaxf(rm, __shfl_xor(rm, 16));
                    rm = fmaxf(rm, __shfl_xor(rm, 32));
                    const float m_new = fmaxf(m_used[mt], rm);
                    const float alpha = fast_exp2(m_used[mt] - m_new);
                    m_used[mt] = m_new;
                    l_part[mt] *= alpha;
#pragma unroll
                    for (int nt = 0; nt < 8; ++nt) oacc[nt][mt] *= alpha;
                }
            }
            bf16x8 pop[MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                float pv[8];
#pragma unroll
                for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                    for (int i = 0; i < 4; ++i) pv[4 * sub + i] = fast_exp2(fmaf(sacc[sub][mt][i], c2, -m_used[mt]));
                if (masked) {
                    // also covers scale == 0, where a masked score can not be told apart by its value
#pragma unroll
                    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            if (!((onmask[mt] >> (16 * sub + 4 * lj + i)) & 1u)) pv[4 * sub + i] = 0.f;
                }
                l_part[mt] += ((pv[0] + pv[1]) + (pv[2] + pv[3])) + ((pv[4] + pv[5]) + (pv[6] + pv[7]));
                u32x4 pk = {pack_bf16(pv[0], pv[1]), pack_bf16(pv[2], pv[3]), pack_bf16(pv[4], pv[5]), pack_bf16(pv[6], pv[7])};
                pop[mt] = __builtin_bit_cast(bf16x8, pk);
            }

            // V tile -> V^T operands (the K operands in the area are dead by now: LDS ops of one wave
            // execute in order)
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int w = e >> 1;
                const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
                u32x4 o;
                o[0] = __builtin_amdgcn_perm(vcur[1][w], vcur[0][w], sel);
                o[1] = __builtin_amdgcn_perm(vcur[3][w], vcur[2][w], sel);
                o[2] = __builtin_amdgcn_perm(vcur[5][w], vcur[4][w], sel);
                o[3] = __builtin_amdgcn_perm(vcur[7][w], vcur[6][w], sel);
                *reinterpret_cast<u32x4 *>(area + 4 * (vst_base + (vst_x ^ e))) = o;
            }
            load_v(PLAIN && !PAGED ? plain_ref(t + KS) : tile_ref(t + KS));
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            // O^T[d][row] += sum_key V[key][d] P[row][key]
#pragma unroll
            for (int nh = 0; nh < 2; ++nh) {
                bf16x8 vop[4];
#pragma unroll
                for (int n4 = 0; n4 < 4; ++n4) {
                    const int nt = 4 * nh + n4;
                    vop[n4] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(area + 4 * (vld_base + nt * 16 + (vld_x ^ ((2 * nt) & 7)))));
                }
#pragma unroll
                for (int n4 = 0; n4 < 4; ++n4)
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
                        oacc[4 * nh + n4][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vop[n4], pop[mt], oacc[4 * nh + n4][mt], 0, 0, 0);
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
        };
        if (COOP) {
            // Tiles alternate between the two register stages / LDS buffers.  The pair loop has no
            // branch around its second half: with one, the wait for a stage's data at the top of
            // the loop would have to cover the path on which no younger loads are in flight, that
            // is, wait for everything.  An odd last tile is handled after the loop.
            // The bulk of a long contiguous prefix goes through the plain step: while t + 4 is
            // still a whole prefix tile of this segment, so are t, t + 1 and the two tiles requested
            // during the pair.
            {
                const int t_plain = min(t_end, L / KT);
                for (; t + 4 < t_plain; t += 2) {
                    tile_step(t, std::integral_constant<int, 0>(), std::true_type());
                    tile_step(t + 1, std::integral_constant<int, 1>(), std::true_type());
                }
            }
            for (; t + 1 < t_end; t += 2) {
                tile_step(t, std::integral_constant<int, 0>(), std::false_type());
                tile_step(t + 1, std::integral_constant<int, 1>(), std::false_type());
            }
            if (t < t_end) tile_step(t, std::integral_constant<int, 0>(), std::false_type());
        } else {
            {
                const int t_plain = min(t_end, L / KT);
                for (; t + KS < t_plain; t += KS) tile_step(t, std::integral_constant<int, 0>(), std::true_type());
            }
            for (; t < t_end; t += KS) tile_step(t, std::integral_constant<int, 0>(), std::false_type());
        }

        // ---- epilogue: merge the key streams.  (m, l) per row through LDS; O in two halves of d:
        // every wave stores its rescaled half as float4 rows [row][68] in its own area, then all
        // threads add up the KS areas of a row group and write the result.
        // The lane indices are re-derived from an opaque copy so that the epilogue's address
        // arithmetic is not hoisted above the tile loop, where it would cost registers (and spill).
        int tid_e = tid;
        asm volatile("" : "+v"(tid_e));
        const int lj_e = (tid_e & 63) >> 4, lc_e = tid_e & 15;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            float lt = l_part[mt];
            lt += __shfl_xor(lt, 16);
            lt += __shfl_xor(lt, 32);
            if (lj_e == 0) { s_m[ks][WROWS * rh + 16 * mt + lc_e] = m_used[mt]; s_l[ks][WROWS * rh + 16 * mt + lc_e] = lt; }
        }
        __syncthreads();
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const int r = WROWS * rh + 16 * mt + lc_e;
            float ms = s_m[0][r];
#pragma unroll
            for (int k2 = 1; k2 < KS; ++k2) ms = fmaxf(ms, s_m[k2][r]);
            const float fsc = exp2f(m_used[mt] - ms);
#pragma unroll
            for (int nt = 0; nt < 8; ++nt) oacc[nt][mt] *= fsc;
        }
        if (tid_e < ROWS) {
            float ms = s_m[0][tid_e];
#pragma unroll
            for (int k2 = 1; k2 < KS; ++k2) ms = fmaxf(ms, s_m[k2][tid_e]);
            float ls = 0.f;
#pragma unroll
            for (int k2 = 0; k2 < KS; ++k2) ls += exp2f(s_m[k2][tid_e] - ms) * s_l[k2][tid_e];
            s_mstar[tid_e] = ms;
            s_linv[tid_e] = direct ? 1.0f / ls : ls;
        }
        const int rows_valid = min(ROWS, p.M - row0);
        float *farea = reinterpret_cast<float *>(area);
#pragma unroll
        for (int half = 0; half < 2; ++half) {
#pragma unroll
            for (int n4 = 0; n4 < 4; ++n4)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    const f32x4 v = oacc[4 * half + n4][mt];       // d = 64 half + 16 n4 + 4 lj + (0..3), row 16 mt + lc
                    *reinterpret_cast<f32x4 *>(farea + (16 * mt + lc_e) * 68 + 16 * n4 + 4 * lj_e) = v;
                }
            __syncthreads();
            // one 16-byte piece per lane, neighbouring lanes neighbouring pieces: every store
            // instruction of the partial covers whole 256-byte runs
            for (int idx = tid_e; idx < rows_valid * 16; idx += NT) {
                const int r = idx >> 4, d4 = idx & 15;
                const int rg = r / WROWS, rl = r % WROWS;
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int k2 = 0; k2 < KS; ++k2)
                    acc += *reinterpret_cast<const f32x4 *>(reinterpret_cast<const float *>(s_big + (rg * KS + k2) * AREA_WORDS) + rl * 68 + 4 * d4);
                const int dcol = 64 * half + 4 * d4;
                if (direct) {
                    const float inv = s_linv[r];
                    const uint2 pk = {pack_bf16(acc[0] * inv, acc[1] * inv), pack_bf16(acc[2] * inv, acc[3] * inv)};
                    const int gr = row0 + r, node = gr / p.G, hh = gr % p.G;
                    uint16_t *ob = static_cast<uint16_t *>(p.out);
                    // outputs and partials are written once and not read again by this kernel: stored
                    // non-temporally they do not sit dirty in L2 until the end-of-kernel write-back
                    __builtin_nontemporal_store((u32x2){pk.x, pk.y}, reinterpret_cast<u32x2 *>(ob + (((size_t)b * p.N + node) * p.H_q + (size_t)g * p.G + hh) * D + dcol));
                } else {
                    __builtin_nontemporal_store(acc, reinterpret_cast<f32x4 *>(p.part_o + (part_row + r) * D + dcol));
                }
            }
            __syncthreads();
        }
        if (!direct && tid_e < rows_valid) {
            p.part_m[part_row + tid_e] = s_mstar[tid_e];
            p.part_l[part_row + tid_e] = s_linv[tid_e];
        }
    }
}

// Merges the chunks of one unit: out = sum_c 2^(m_c - m*) O_c / sum_c 2^(m_c - m*) l_c.
// Blocks with blockIdx.x >= nx_combine carry the walk of a verification that ran before this
// launch on the same stream (one thread per sequence), when the caller asked for that.
__global__ __launch_bounds__(256) void tree_attn_combine_kernel(AttnParams p, int nx_combine, WalkParams w)
{
    constexpr int D = 128;
    if ((int)blockIdx.x >= nx_combine) {
        if (blockIdx.y == 0 && blockIdx.z == 0) {
            const int wb = ((int)blockIdx.x - nx_combine) * 256 + (int)threadIdx.x;
            if (wb < w.B) walk_sequence(w, wb);
        }
        return;
    }
    const int g = blockIdx.y, b = blockIdx.z;
    int L = p.prefix_len[b];
    L = max(0, min(L, p.L_stride));
    const int total_tiles = (L + KT - 1) / KT + p.tiles_tree;
    int n_chunks, seg;
    split_tiles(total_tiles, p.chunk_tiles, p.split_bias, &n_chunks, &seg);
    n_chunks = (total_tiles + seg - 1) / seg;      // segments that are not empty
    if (n_chunks <= 1) return;      // the attention kernel wrote the output itself
    const int r = blockIdx.x * 8 + (threadIdx.x >> 5);
    const int d4 = threadIdx.x & 31;        // 16-byte piece of the row
    if (r >= p.M) return;
    const size_t base = (((size_t)b * p.H_kv + g) * p.n_chunks_max) * (size_t)p.R + r;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    float ls = 0.f;
    // Up to eight chunks (the usual case) every load is issued before the first use: one memory
    // round trip instead of one per chunk.  Slots past n_chunks re-read chunk 0 (a cache hit) with
    // weight zero, so the loads stay unconditional; two sizes keep that waste below a factor of two.
    auto merge_upfront = [&](auto maxc) __attribute__((always_inline)) {
        constexpr int MAXC = decltype(maxc)::value;
        float mc[MAXC], lc[MAXC];
        f32x4 oc[MAXC];
#pragma unroll
        for (int c = 0; c < MAXC; ++c) {
            const bool on = c < n_chunks;
            const size_t u = base + (size_t)(on ? c : 0) * p.R;
            mc[c] = on ? p.part_m[u] : M_INIT;
            lc[c] = on ? p.part_l[u] : 0.f;
            oc[c] = *reinterpret_cast<const f32x4 *>(p.part_o + u * D + 4 * d4);
        }
        float ms = mc[0];
#pragma unroll
        for (int c = 1; c < MAXC; ++c) ms = fmaxf(ms, mc[c]);
#pragma unroll
        for (int c = 0; c < MAXC; ++c) {
            const float fsc = (c < n_chunks) ? exp2f(mc[c] - ms) : 0.f;
            ls += fsc * lc[c];
            acc += fsc * oc[c];
        }
    };
    if (n_chunks <= 4) {
        merge_upfront(std::integral_constant<int, 4>());
    } else if (n_chunks <= 8) {
        merge_upfront(std::integral_constant<int, 8>());
    } else {
        float ms = M_INIT;
        for (int c = 0; c < n_chunks; ++c) ms = fmaxf(ms, p.part_m[base + (size_t)c * p.R]);
        for (int c = 0; c < n_chunks; ++c) {
            const size_t u = base + (size_t)c * p.R;
            const float fsc = exp2f(p.part_m[u] - ms);
            ls += fsc * p.part_l[u];
            acc += fsc * *reinterpret_cast<const f32x4 *>(p.part_o + u * D + 4 * d4);
        }
    }
    const float inv = 1.0f / ls;
    const uint2 pk = {pack_bf16(acc[0] * inv, acc[1] * inv), pack_bf16(acc[2] * inv, acc[3] * inv)};
    const int node = r / p.G, hh = r % p.G;
    uint16_t *ob = static_cast<uint16_t *>(p.out);
    __builtin_nontemporal_store((u32x2){pk.x, pk.y}, reinterpret_cast<u32x2 *>(ob + (((size_t)b * p.N + node) * p.H_q + (size_t)g * p.G + hh) * D + 4 * d4));
}

// ------------------------------------------------------------------ generic path
// One 256-thread workgroup per (sequence, node, query head).  Keys are taken 256 at
// a time: thread t scores key t (dot product over d on the vector ALU), the running
// max is a wavefront-shuffle + LDS reduction, the weights go to LDS, and thread t
// (t < d) accumulates output column t over the 256 keys.
template <typename T>
__device__ __forceinline__ float load_as_float(const T *p, size_t i);
template <>
__device__ __forceinline__ float load_as_float<float>(const float *p, size_t i) { return p[i]; }
template <>
__device__ __forceinline__ float load_as_float<uint16_t>(const uint16_t *p, size_t i) { return bf16_bits_to_float(p[i]); }

template <typename T>
__device__ __forceinline__ void store_from_float(T *p, size_t i, float v);
template <>
__device__ __forceinline__ void store_from_float<float>(float *p, size_t i, float v) { p[i] = v; }
template <>
__device__ __forceinline__ void store_from_float<uint16_t>(uint16_t *p, size_t i, float v)
{
    p[i] = (uint16_t)(pack_bf16(v, 0.f) & 0xffffu);
}

template <typename T>
__global__ __launch_bounds__(256) void tree_attn_generic_kernel(AttnParams p)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int h = blockIdx.x, node = blockIdx.y, b = blockIdx.z;
    const int g = h / p.G, d = p.d;
    __shared__ float s_q[MCSD_MAX_HEAD_DIM];
    __shared__ float s_p[256];
    __shared__ float s_red[4];
    __shared__ uint32_t s_anc[MCSD_MAX_NODES][4];
    __shared__ int s_parent[MCSD_MAX_NODES];

    build_ancestor_masks(p.parent + (p.parent_per_seq ? (size_t)b * (p.N - p.root_row) : 0), p.N, p.root_row, s_anc, s_parent);
    const T *qp = static_cast<const T *>(p.q) + (((size_t)b * p.N + node) * p.H_q + h) * (size_t)d;
    for (int c = tid; c < d; c += 256) s_q[c] = load_as_float<T>(qp, c);
    __syncthreads();

    int L = p.prefix_len[b];
    L = max(0, min(L, p.L_stride));
    const size_t kv_head = (size_t)b * p.H_kv + g;
    const bool paged = p.block_table != nullptr;
    const T *kpre = static_cast<const T *>(p.k_prefix) + (paged ? 0 : kv_head * (size_t)p.L_stride * d);
    const T *vpre = static_cast<const T *>(p.v_prefix) + (paged ? 0 : kv_head * (size_t)p.L_stride * d);
    // row index (in units of d elements) of logical prefix row r inside kpre / vpre
    auto prefix_row = [&](int r) -> size_t {
        if (!paged) return (size_t)r;
        int blk = p.block_table[(size_t)b * p.max_pages + r / p.page_size];
        blk = min(max(blk, 0), p.n_pages - 1);      // an entry outside the pool never leaves it
        return ((size_t)blk * p.H_kv + g) * (size_t)p.page_size + (size_t)(r % p.page_size);
    };
    const T *ktre = static_cast<const T *>(p.k_tree) + kv_head * (size_t)p.N * d;
    const T *vtre = static_cast<const T *>(p.v_tree) + kv_head * (size_t)p.N * d;
    const int n_keys = L + p.N;

    float m_run = M_INIT, l_run = 0.f, o_acc = 0.f;      // o_acc: output column tid (tid < d)
    for (int k0 = 0; k0 < n_keys; k0 += 256) {
        const int key = k0 + tid;
        float s = -INFINITY;
        if (key < n_keys) {
            bool on = true;
            const T *kr;
            if (key < L) kr = kpre + prefix_row(key) * d;
            else {
                const int a = key - L;
                on = (s_anc[node][a >> 5] >> (a & 31)) & 1u;
                kr = ktre + (size_t)a * d;
            }
            if (on) {
                float acc = 0.f;
                for (int c = 0; c < d; ++c) acc += s_q[c] * load_as_float<T>(kr, c);
                s = acc * p.scale_log2;
            }
        }
        float cm = s;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) cm = fmaxf(cm, __shfl_xor(cm, o));
        if (lane == 0) s_red[wave] = cm;
        __syncthreads();
        cm = fmaxf(fmaxf(s_red[0], s_red[1]), fmaxf(s_red[2], s_red[3]));
        const float m_new = fmaxf(m_run, cm);
        const float alpha = exp2f(m_run - m_new);
        const float pw = exp2f(s - m_new);          // 0 for masked / out-of-range keys
        s_p[tid] = pw;
        __syncthreads();
        float ps = 0.f;
        const int cnt = min(256, n_keys - k0);
        if (tid < d) {
            float acc = 0.f;
            for (int j = 0; j < cnt; ++j) {
                const int kj = k0 + j;
                const T *vr = (kj < L) ? vpre + prefix_row(kj) * d : vtre + (size_t)(kj - L) * d;
                acc += s_p[j] * load_as_float<T>(vr, tid);
            }
            o_acc = o_acc * alpha + acc;
        }
        for (int j = 0; j < cnt; ++j) ps += s_p[j];
        l_run = l_run * alpha + ps;
        m_run = m_new;
        __syncthreads();
    }
    if (tid < d) {
        T *op = static_cast<T *>(p.out) + (((size_t)b * p.N + node) * p.H_q + h) * (size_t)d;
        store_from_float<T>(op, tid, o_acc / l_run);
    }
}

// Launch-plan overrides of mcsd_attn_plan_override (0 = automatic), process-wide.
std::atomic<int> g_force_variant{0}, g_force_chunk_tiles{0}, g_force_target_wgs{0};

}  // namespace

bool make_attn_plan(const mcsd_attn_desc &d, AttnPlan *plan)
{
    AttnPlan pl = {};
    const int G = d.H_q / d.H_kv;
    const int n_rows_tree = d.N + (d.root_row ? 1 : 0);      // rows of the tree block
    pl.rows_per_kv = n_rows_tree * G;
    pl.use_mfma = (d.dtype == MCSD_DTYPE_BF16 && d.d == 128);
    if (!pl.use_mfma) {
        if (d.d > MCSD_MAX_HEAD_DIM) return false;
        pl.ws_bytes = 0;
        *plan = pl;
        return true;
    }
    // Kernel variant (4 waves, two workgroups per CU): 0 = 32 rows x 4 key streams for
    // rows_per_kv <= 32, 1 = 2 x 32 rows x 2 key streams up to 64 rows, 2 = 4 x 32 rows on one
    // key stream with tiles shared through LDS beyond that (several row tiles per KV head:
    // the matrix cores are the limit there, and the shared tiles cut the per-wave staging work).
    pl.variant = pl.rows_per_kv <= 32 ? 0 : (pl.rows_per_kv <= 64 ? 1 : 2);
    {
        const int forced_variant = g_force_variant.load();     // 1-based, 0 = automatic
        if (forced_variant >= 1 && forced_variant <= 3) pl.variant = forced_variant - 1;
    }
    pl.row_tile = 32 << pl.variant;
    const int key_streams = 4 >> pl.variant;
    pl.n_row_tiles = (pl.rows_per_kv + pl.row_tile - 1) / pl.row_tile;
    pl.tiles_prefix_max = (d.L_stride + KT - 1) / KT;
    pl.tiles_tree = (n_rows_tree + KT - 1) / KT;
    const long total_max = pl.tiles_prefix_max + pl.tiles_tree;
    const long units = (long)d.B * d.H_kv * pl.n_row_tiles;
    // Every segment pays a fixed prologue (Q, first tiles) and epilogue (merge, possibly one
    // [rows][d] fp32 partial written and read back by the combine kernel), which runs shorter
    // than 6 tiles per key stream do not amortise (measured).
    const long min_run = 6 * key_streams;

    // Workgroups per launch if every sequence had the maximum length (the CUs hold 512 at a time).
    // More, shorter segments balance the end of the launch better but every segment of a split
    // unit costs one fp32 partial written and read back; 1024 measured best both where the
    // kernel is HBM-bound (that traffic competes with the cache stream) and where the matrix
    // cores are the limit (768 .. 1536 within 2 %; beyond that the merge kernel grows faster
    // than the attention kernel shrinks).
    const int forced_target = g_force_target_wgs.load();
    const long target_wgs = forced_target > 0 ? forced_target : 1024;
    long chunk = (total_max * units + target_wgs - 1) / target_wgs;
    chunk = ((chunk + key_streams - 1) / key_streams) * key_streams;
    if (chunk < min_run) chunk = min_run;
    const int forced = g_force_chunk_tiles.load();
    if (forced > 0) chunk = forced;
    if (chunk > total_max) chunk = total_max;
    pl.chunk_tiles = (int)chunk;
    pl.n_chunks_max = (int)((total_max + chunk - 1) / chunk);
    pl.partial_stride_rows = (size_t)pl.n_row_tiles * pl.row_tile;
    if (pl.n_chunks_max > 1) {
        size_t elems = (size_t)d.B * d.H_kv * pl.n_chunks_max * pl.partial_stride_rows * (size_t)(d.d + 2);
        pl.ws_bytes = (elems * sizeof(float) + 255) & ~(size_t)255;
    } else {
        pl.ws_bytes = 0;
    }
    if ((long)pl.n_chunks_max * pl.n_row_tiles + 256L > 65535L || d.B > 65535) return false;     // (+ rows that may carry a walk)
    *plan = pl;
    return true;
}

int32_t attn_plan_override(int variant, int chunk_tiles, int target_wgs)
{
    if (variant < 0 || variant > 3 || chunk_tiles < 0 || target_wgs < 0) return MCSD_E_SHAPE;
    g_force_variant.store(variant);
    g_force_chunk_tiles.store(chunk_tiles);
    g_force_target_wgs.store(target_wgs);
    return MCSD_OK;
}

int32_t launch_tree_attn(const mcsd_attn_desc &d, const mcsd_attn_bufs &b, const AttnPlan &plan,
                         hipStream_t stream, const mcsd_paged_kv *paged, int phases, const WalkParams *tail_walk)
{
    AttnParams p = {};
    if (paged) {
        p.block_table = paged->block_table; p.page_size = paged->page_size;
        p.n_pages = paged->n_pages; p.max_pages = paged->max_pages_per_seq;
    }
    p.q = b.q; p.k_prefix = b.k_prefix; p.v_prefix = b.v_prefix; p.k_tree = b.k_tree; p.v_tree = b.v_tree;
    p.prefix_len = b.prefix_len; p.parent = b.parent; p.out = b.out;
    p.root_row = d.root_row ? 1 : 0;
    p.B = d.B; p.N = d.N + p.root_row; p.H_q = d.H_q; p.H_kv = d.H_kv; p.G = d.H_q / d.H_kv; p.d = d.d;
    p.L_stride = d.L_stride; p.M = plan.rows_per_kv; p.parent_per_seq = d.parent_per_seq; p.dtype = d.dtype;
    p.scale_log2 = d.scale * LOG2E_F;
    hipError_t e;
    if (!plan.use_mfma) {
        if (d.H_q > 2147483647 || d.B > 65535) { set_error("attn: grid too large"); return MCSD_E_UNSUPPORTED; }
        dim3 grid(d.H_q, p.N, d.B), block(256);
        if (d.dtype == MCSD_DTYPE_FP32)
            launch_kernel(K_ATTN_GENERIC, tree_attn_generic_kernel<float>, grid, block, stream, p);
        else
            launch_kernel(K_ATTN_GENERIC, tree_attn_generic_kernel<uint16_t>, grid, block, stream, p);
        e = hipGetLastError();
        if (e != hipSuccess) { set_error("tree_attn_generic launch failed: %s", hipGetErrorString(e)); return MCSD_E_HIP; }
        return MCSD_OK;
    }
    p.n_row_tiles = plan.n_row_tiles; p.chunk_tiles = plan.chunk_tiles; p.n_chunks_max = plan.n_chunks_max;
    p.tiles_tree = plan.tiles_tree; p.R = (int)plan.partial_stride_rows;
    p.split_bias = plan.chunk_tiles / 2;
    if (plan.ws_bytes > 0) {
        const size_t rows = (size_t)d.B * d.H_kv * plan.n_chunks_max * plan.partial_stride_rows;
        float *ws = static_cast<float *>(b.workspace);
        p.part_o = ws;
        p.part_m = ws + rows * d.d;
        p.part_l = p.part_m + rows;
    }
    if (phases & ATTN_PHASE_MAIN) {
        // an unsplit attention has no merge launch to carry the walk: it rides on this one
        WalkParams mw = {};
        int walk_rows = 0;
        if (tail_walk && plan.n_chunks_max == 1) { mw = *tail_walk; walk_rows = (mw.B + 255) / 256; }
        const dim3 grid(d.H_kv, plan.n_chunks_max * plan.n_row_tiles + walk_rows, d.B);
        if (paged) {
            if (plan.variant == 0) launch_kernel(K_ATTN_MFMA, tree_attn_mfma_kernel<1, 4, true>, grid, dim3(256), stream, p, mw);
            else if (plan.variant == 1) launch_kernel(K_ATTN_MFMA, tree_attn_mfma_kernel<2, 2, true>, grid, dim3(256), stream, p, mw);
            else launch_kernel(K_ATTN_MFMA, tree_attn_mfma_kernel<4, 1, true, true>, grid, dim3(256), stream, p, mw);
        } else {
            if (plan.variant == 0) launch_kernel(K_ATTN_MFMA, tree_attn_mfma_kernel<1, 4, false>, grid, dim3(256), stream, p, mw);
            else if (plan.variant == 1) launch_kernel(K_ATTN_MFMA, tree_attn_mfma_kernel<2, 2, false>, grid, dim3(256), stream, p, mw);
            else launch_kernel(K_ATTN_MFMA, tree_attn_mfma_kernel<4, 1, false, true>, grid, dim3(256), stream, p, mw);
        }
        e = hipGetLastError();
        if (e != hipSuccess) { set_error("tree_attn_mfma launch failed: %s", hipGetErrorString(e)); return MCSD_E_HIP; }
    }
    if ((phases & ATTN_PHASE_COMBINE) && plan.n_chunks_max > 1) {
        const int nx = (plan.rows_per_kv + 7) / 8;
        WalkParams w = {};
        int walk_blocks = 0;
        if (tail_walk) { w = *tail_walk; walk_blocks = (w.B + 255) / 256; }
        dim3 cgrid(nx + walk_blocks, d.H_kv, d.B);
        launch_kernel(K_ATTN_COMBINE, tree_attn_combine_kernel, cgrid, dim3(256), stream, p, nx, w);
        e = hipGetLastError();
        if (e != hipSuccess) { set_error("tree_attn_combine launch failed: %s", hipGetErrorString(e)); return MCSD_E_HIP; }
    }
    return MCSD_OK;
}

}  // namespace mcsd
