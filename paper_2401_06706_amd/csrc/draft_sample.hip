// Draft-side candidate sampling on gfx950 (Sec. 3.1 of the paper; q-bar of Eq. (1) when the
// candidates are drawn without replacement).
//
// One workgroup owns one row of the tree that has children.  The draft logit row is read
// from HBM once with 128-bit loads and stays in registers; after one max and one exp/sum pass
// the k draws are k inverse-CDF searches over the resident weights (two-level, fp64).  Without
// replacement the drawn token's weight is zeroed in its register and subtracted from the
// running mass, which is q-bar of Eq. (1) without a renormalising pass: the search compares
// against u times the remaining mass.  At temperature 0 the candidates are the k largest
// logits: k rounds of a workgroup arg max (lowest id on ties), each removing its winner.
#include <math.h>

#include "mcsd_internal.h"
#include "vocab_row.h"

namespace mcsd {
namespace {

using namespace vocab;

constexpr float LOG2E_F = 1.44269504088896340736f;

struct DraftParams {
    int B, N, V, P, variant, per_seq;
    float eps;
    const float *draft_logits;
    const int32_t *q_row, *parent;
    const float *u_draw, *temperature;
    int32_t *cand_tok;
    uint32_t *flags;
};

template <int ITEMS, int VT, bool ALIGNED>
__global__ __launch_bounds__(VT) void draft_rows_kernel(DraftParams p)
{
    constexpr int NWAVES = VT / 64;
    const int row = blockIdx.x, b = blockIdx.y;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int N = p.N, V = p.V;

    __shared__ double s_red[NWAVES];
    __shared__ double s_seg[4 * NWAVES * ITEMS];
    __shared__ double s_tot[ITEMS];
    __shared__ float s_redf[NWAVES];
    __shared__ unsigned long long s_mask[2];
    __shared__ int s_kids[MCSD_MAX_NODES];
    __shared__ int s_k;
    __shared__ int s_int[4];
    __shared__ uint32_t s_flag;
    __shared__ float s_removed;
    __shared__ float s_bestv[NWAVES];
    __shared__ int s_besti[NWAVES];

    // The row is requested before it is known whether this tree row has children: in a
    // well-formed input q_row marks exactly the rows that do.
    const int qr = p.q_row[(p.per_seq ? (size_t)b * (1 + N) : 0) + row];
    const int32_t *parent = p.parent + (p.per_seq ? (size_t)b * N : 0);
    const bool have_q = qr >= 0 && qr < p.P;
    float4 a[ITEMS];
    if (have_q) {
        load_row<ITEMS, VT, ALIGNED>(p.draft_logits + ((size_t)b * p.P + qr) * (size_t)V, V, a);
    } else {
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) a[i] = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
    }
    const float T = p.temperature[b];

    // children of this row, ascending node id = sampling order
    if (t < 128) {
        const bool f = (t < N) && (parent[t] == row - 1);
        const unsigned long long m = __ballot(f);
        if (lane == 0) s_mask[wave] = m;
    }
    __syncthreads();
    if (t == 0) {
        int k = 0;
        for (int w = 0; w < 2; ++w) {
            unsigned long long m = s_mask[w];
            while (m) {
                s_kids[k++] = w * 64 + (__ffsll((long long)m) - 1);
                m &= m - 1;
            }
        }
        s_k = k;
    }
    __syncthreads();
    const int k = s_k;
    if (k == 0) return;
    if (!have_q || k > V) {
        // children without a draft row (or more children than tokens): reported, nothing drawn
        if (t < k) {
            p.cand_tok[(size_t)b * N + s_kids[t]] = -1;
            p.flags[(size_t)b * N + s_kids[t]] = (uint32_t)MCSD_FLAG_BAD_TREE;
        }
        return;
    }

    if (T == 0.f) {
        // largest value of the workgroup and the lowest token id that holds it, in every thread
        auto block_argmax = [&](float &bv, int &bi) __attribute__((always_inline)) {
            wave_argmax(bv, bi);
            if (lane == 0) { s_bestv[wave] = bv; s_besti[wave] = bi; }
            __syncthreads();
            bv = s_bestv[0]; bi = s_besti[0];
            for (int w = 1; w < NWAVES; ++w)
                if (s_bestv[w] > bv || (s_bestv[w] == bv && s_besti[w] < bi)) { bv = s_bestv[w]; bi = s_besti[w]; }
            __syncthreads();
        };
        for (int i = 0; i < k; ++i) {
            // A thread meets its elements in ascending token order, so a strict comparison keeps
            // the lowest id among equal values; it never picks a logit of -inf (nor the -inf
            // padding past V), which is only right while something finite is left ...
            float bv = -INFINITY;
            int bi = 0x7fffffff;
#pragma unroll
            for (int j = 0; j < ITEMS; ++j) {
                const int e = 4 * (t + VT * j);
                const float v[4] = {a[j].x, a[j].y, a[j].z, a[j].w};
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (v[c] > bv) { bv = v[c]; bi = e + c; }
            }
            block_argmax(bv, bi);
            if (bi == 0x7fffffff) {
                // ... otherwise (every thread sees the same result) the scan is repeated with
                // -inf allowed to win, inside the row only
                bv = -INFINITY;
#pragma unroll
                for (int j = 0; j < ITEMS; ++j) {
                    const int e = 4 * (t + VT * j);
                    const float v[4] = {a[j].x, a[j].y, a[j].z, a[j].w};
#pragma unroll
                    for (int c = 0; c < 4; ++c)
                        if (e + c < V && (v[c] > bv || (v[c] == bv && e + c < bi))) { bv = v[c]; bi = e + c; }
                }
                block_argmax(bv, bi);
            }
            // nothing comparable left (only NaN logits remain): reported, token 0 handed out
            const bool none = (bi == 0x7fffffff);
            if (none) bi = 0;
            if (t == 0) {
                p.cand_tok[(size_t)b * N + s_kids[i]] = bi;
                p.flags[(size_t)b * N + s_kids[i]] = none ? (uint32_t)MCSD_FLAG_NONFINITE : 0u;
            }
            // the winner leaves the row (ids are unique, one thread owns it): a NaN never wins a
            // comparison, while a logit of -inf still can once everything above it is taken
            const float gone = __int_as_float(0x7fc00000);
#pragma unroll
            for (int j = 0; j < ITEMS; ++j) {
                const int e = 4 * (t + VT * j);
                if (bi == e) a[j].x = gone;
                if (bi == e + 1) a[j].y = gone;
                if (bi == e + 2) a[j].z = gone;
                if (bi == e + 3) a[j].w = gone;
            }
        }
        return;
    }

    const float c2 = (1.0f / T) * LOG2E_F;
    const float m = block_max<NWAVES>(row_max<ITEMS>(a), s_redf);
    double Z = block_sum<NWAVES>(row_exp<ITEMS>(a, m, c2), s_red);       // a = e_q, Z = its sum
    const bool finite = (Z > 0.0) && (Z < INFINITY);
    // segment totals once; the k searches reuse them (kept in step when a token is removed)
    cdf_segments<ITEMS, VT>(a, s_seg, s_tot);
    for (int i = 0; i < k; ++i) {
        const int node = s_kids[i];
        if (t == 0) s_flag = 0u;
        __syncthreads();
        int x = 0;
        const bool ok = finite && Z > 0.0;
        if (ok) {
            const double u = (double)p.u_draw[(size_t)b * N + node];
            x = cdf_search<ITEMS, VT>(a, Z, u, (double)p.eps, s_red, s_tot, s_int, &s_flag);
            if (x < 0 || x >= V) x = V - 1;
        }
        if (t == 0) {
            uint32_t fl = (s_flag & MCSD_FLAG_NEAR_TIE_ENDPOINT) ? (uint32_t)MCSD_FLAG_NEAR_TIE_DRAW : 0u;
            if (!ok) fl |= (uint32_t)MCSD_FLAG_NONFINITE;
            p.cand_tok[(size_t)b * N + node] = x;
            p.flags[(size_t)b * N + node] = fl;
        }
        if (p.variant == MCSD_WITHOUT_REPLACEMENT && i + 1 < k) {
            // q-bar of Eq. (1): the drawn token's weight leaves its register, its segment and the mass
#pragma unroll
            for (int j = 0; j < ITEMS; ++j) {
                const int e = 4 * (t + VT * j);
                if ((x >> 2) == (e >> 2)) {
                    float w = 0.f;
                    if (x == e) { w = a[j].x; a[j].x = 0.f; }
                    if (x == e + 1) { w = a[j].y; a[j].y = 0.f; }
                    if (x == e + 2) { w = a[j].z; a[j].z = 0.f; }
                    if (x == e + 3) { w = a[j].w; a[j].w = 0.f; }
                    s_tot[j] -= (double)w;
                    s_removed = w;
                }
            }
            __syncthreads();
            Z -= (double)s_removed;
        }
        __syncthreads();
    }
}

template <int ITEMS, int VT>
void launch_rows(const DraftParams &p, hipStream_t stream)
{
    dim3 grid(1 + p.N, p.B), block(VT);
    if (p.V % 4 == 0)
        launch_kernel(K_DRAFT_ROWS, draft_rows_kernel<ITEMS, VT, true>, grid, block, stream, p);
    else
        launch_kernel(K_DRAFT_ROWS, draft_rows_kernel<ITEMS, VT, false>, grid, block, stream, p);
}

}  // namespace

int32_t launch_draft_sample(const mcsd_draft_desc &d, const mcsd_draft_bufs &b, hipStream_t stream)
{
    DraftParams p;
    p.B = d.B; p.N = d.N; p.V = d.V; p.P = d.P; p.variant = d.variant; p.eps = d.near_tie_eps; p.per_seq = d.parent_per_seq;
    p.draft_logits = b.draft_logits; p.q_row = b.q_row; p.parent = b.parent;
    p.u_draw = b.u_draw; p.temperature = b.temperature; p.cand_tok = b.cand_tok; p.flags = b.flags;
    // the row stays in registers: 1024 threads up to 8192 tokens, 512 threads with more
    // registers each beyond that (a 1024-thread workgroup is capped at 128 registers per thread)
    if (d.V <= 4096) launch_rows<1, 1024>(p, stream);
    else if (d.V <= 8192) launch_rows<2, 1024>(p, stream);
    else if (d.V <= 16384) launch_rows<8, 512>(p, stream);
    else if (d.V <= 32768) launch_rows<16, 512>(p, stream);
    else launch_rows<32, 512>(p, stream);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_error("draft_rows launch failed: %s", hipGetErrorString(e));
        return MCSD_E_HIP;
    }
    return MCSD_OK;
}

}  // namespace mcsd
