// Multi-candidate speculative sampling on gfx950: Algorithm 1 (with replacement),
// Algorithm 2 (without replacement), the endpoint draws and the root-to-leaf walk.
//
// One workgroup owns one row of the tree (the root or a node).
//
// verify_rows_kernel (vocabularies up to 32768): both logit rows of the node are read from HBM
// exactly once with 128-bit buffer loads and stay in registers for all k sequential
// accept/reject rounds; every round is one elementwise pass over the resident data plus one
// block reduction.  1024 threads up to 16384 tokens, 512 threads (twice the registers) beyond.
//
// verify_rows_stream_kernel (up to 65536): only the target row stays in registers, as the
// unnormalised residual a(x).  The draft row is streamed: once from HBM for its maximum, again
// (from the caches) for the exponentials and their sum, and once more for every rejection,
// where the update a := max(0, a - beta e_q) needs e_q(x) = exp((z_q(x) - max) / T),
// recomputed on the fly.  Algorithm 2's removal of a rejected token from q needs no pass
// there: that token's residual is already 0 and stays 0 whatever is subtracted from it later,
// so only Z_q changes, by exactly the fp32 weight of the token.
//
// Instead of renormalising after each rejection the kernels carry an
// unnormalised residual a(x) and its sum A (p-hat = a / A), and the unnormalised
// draft weights e_q(x) with the running mass Z_q of the tokens not yet removed
// (q-bar = e_q / Z_q).  Algorithm 1/2's update p := max(0, p - q) / sum(...) then
// reads a := max(0, a - (A / Z_q) e_q), A := sum a, and the normaliser the paper
// divides by (the probability of the rejection, Appendix A) is A_new / A_old.
//
// The handful of numbers that decide an accept test - a(x), e_q(x) at the k
// candidate tokens - are tracked separately in fp64 by one thread per candidate,
// so that the comparison u <= min(1, p/q) is taken at far better than the 1e-6
// near-tie band; vocabulary-wide passes are fp32 with fp64 accumulation.
#include <math.h>
#include <stdlib.h>

#include "mcsd_internal.h"
#include "vocab_row.h"

namespace mcsd {
namespace {

using namespace vocab;

constexpr float LOG2E_F = 1.44269504088896340736f;

struct VerifyParams {
    int B, N, V, P, variant, gamma_max, per_seq;
    float eps;
    const float *target_logits, *draft_logits;
    const int32_t *q_row, *parent, *cand_tok;
    const float *u_accept, *u_endpoint, *temperature;
    int32_t *n_accepted, *accepted_path, *out_tokens, *acc_child, *endpoint;
    float *ratio;
    uint32_t *flags;
    float *residual_out;
};

// 2^x in fp64 for x <= 0 (one thread per candidate token evaluates two of these): x = n + f with
// |f| <= 1/2, 2^f = exp(f ln 2) by its Taylor series to degree 13 (|f ln 2| <= 0.35: truncation
// below 1e-17), scaled by 2^n.  Arguments below -1000 return 0.
__device__ __forceinline__ double exp2_neg(double x)
{
    if (!(x > -1000.0)) return 0.0;
    const double n = rint(x);
    const double y = (x - n) * 0.69314718055994530942;
    double r = 1.0 / 6227020800.0;
    r = fma(r, y, 1.0 / 479001600.0);
    r = fma(r, y, 1.0 / 39916800.0);
    r = fma(r, y, 1.0 / 3628800.0);
    r = fma(r, y, 1.0 / 362880.0);
    r = fma(r, y, 1.0 / 40320.0);
    r = fma(r, y, 1.0 / 5040.0);
    r = fma(r, y, 1.0 / 720.0);
    r = fma(r, y, 1.0 / 120.0);
    r = fma(r, y, 1.0 / 24.0);
    r = fma(r, y, 1.0 / 6.0);
    r = fma(r, y, 0.5);
    r = fma(r, y, 1.0);
    r = fma(r, y, 1.0);
    return ldexp(r, (int)n);
}


// The arguments of the kernel, read again from the kernel-argument segment through a pointer the
// compiler can not see through.  Used where an argument is needed late in the kernel: kept in
// scalar registers from the start it would be spilled around the vocabulary passes.
__device__ __forceinline__ VerifyParams reload_params()
{
    typedef const uint32_t __attribute__((address_space(4))) *kernarg_words;
    kernarg_words pk = (kernarg_words)__builtin_amdgcn_kernarg_segment_ptr();      // the only argument
    asm volatile("" : "+s"(pk));
    union { VerifyParams params; uint32_t words[sizeof(VerifyParams) / 4]; } copy;
#pragma unroll
    for (int i = 0; i < (int)(sizeof(VerifyParams) / 4); ++i) copy.words[i] = pk[i];
    return copy.params;
}

// The residual row scaled by s, stored through a buffer resource (stores past the end of the row
// are dropped).  The offset of a piece goes into the per-thread offset, not into the scalar
// offset field: with a scalar register there, the compiler inserts no wait between a 128-bit
// store and the next write to its data registers, and on this chip the store then sent the
// next piece's values for some lanes (seen as wrong residuals, in different places from run to run).
template <int ITEMS, int VT, bool ALIGNED>
__device__ __forceinline__ void store_residual(float *dst, int V, const float4 (&a)[ITEMS], float s)
{
    const __amdgpu_buffer_rsrc_t rs_out = row_resource(dst, V);
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        const int off = threadIdx.x * 16 + i * (VT * 16);
        if (ALIGNED) {
            const u32x4 v = {__float_as_uint(a[i].x * s), __float_as_uint(a[i].y * s), __float_as_uint(a[i].z * s), __float_as_uint(a[i].w * s)};
            __builtin_amdgcn_raw_buffer_store_b128(v, rs_out, off, 0, 0);
        } else {
            __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(a[i].x * s), rs_out, off, 0, 0);
            __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(a[i].y * s), rs_out, off + 4, 0, 0);
            __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(a[i].z * s), rs_out, off + 8, 0, 0);
            __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(a[i].w * s), rs_out, off + 12, 0, 0);
        }
    }
}

// One pass over a logit row that is not held in registers: thread t meets the same elements
// as in a resident row (float4 number t + VT i for i = 0 .. ITEMS-1, -inf past V), in chunks of
// CH pieces; f(i, values) is called in ascending i.  DOUBLE: two chunks are in flight, the next
// one is requested before the current one is used; otherwise a chunk is requested when the
// previous one has been used.  In both cases the scheduler may not move requests further ahead
// than that (it would, at the price of spills).
template <int ITEMS, int VT, bool ALIGNED, bool NONTEMPORAL, int CHUNK, bool DOUBLE, typename F>
__device__ __forceinline__ void stream_row(__amdgpu_buffer_rsrc_t rs, int V, F &&f)
{
    constexpr int CH = ITEMS < CHUNK ? ITEMS : CHUNK;
    float4 cur[CH], nxt[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c) cur[c] = load_row_piece<VT, ALIGNED, NONTEMPORAL>(rs, c, V, threadIdx.x);
#pragma unroll
    for (int i0 = 0; i0 < ITEMS; i0 += CH) {
        if (DOUBLE && i0 + CH < ITEMS) {
#pragma unroll
            for (int c = 0; c < CH; ++c) nxt[c] = load_row_piece<VT, ALIGNED, NONTEMPORAL>(rs, i0 + CH + c, V, threadIdx.x);
        }
#pragma unroll
        for (int c = 0; c < CH; ++c) f(i0 + c, cur[c]);
        __builtin_amdgcn_sched_barrier(0);
        if (i0 + CH < ITEMS) {
#pragma unroll
            for (int c = 0; c < CH; ++c) cur[c] = DOUBLE ? nxt[c] : load_row_piece<VT, ALIGNED, NONTEMPORAL>(rs, i0 + CH + c, V, threadIdx.x);
        }
    }
}

// e_q of four logits, bit for bit what every pass (and the thread that tracks a candidate
// token) computes: subtraction first, then the scale, then v_exp_f32.
__device__ __forceinline__ float4 exp_weights(const float4 &z, float m, float c)
{
    return make_float4(__builtin_amdgcn_exp2f((z.x - m) * c), __builtin_amdgcn_exp2f((z.y - m) * c),
                       __builtin_amdgcn_exp2f((z.z - m) * c), __builtin_amdgcn_exp2f((z.w - m) * c));
}

template <int ITEMS, int VT, bool ALIGNED>
__global__ __launch_bounds__(VT) __attribute__((amdgpu_waves_per_eu(ITEMS <= 16 ? 4 : 2, ITEMS <= 16 ? 4 : 2)))
void verify_rows_stream_kernel(VerifyParams p)
{
    constexpr int NWAVES = VT / 64;
    constexpr int PASS_CHUNK = 4;           // pieces of the draft row requested together while the target row is resident
    constexpr bool PASS_DOUBLE = true;
    const int row = blockIdx.x;
    int b = blockIdx.y;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int N = p.N, V = p.V;

    __shared__ double s_red[NWAVES];
    __shared__ double s_red2[NWAVES];
    __shared__ double s_seg[4 * NWAVES * ITEMS + ITEMS];
    __shared__ float s_redf[NWAVES];
    __shared__ float s_redf2[NWAVES];
    __shared__ unsigned long long s_mask[2];
    __shared__ int s_kids[MCSD_MAX_NODES];
    __shared__ int s_k;
    __shared__ int s_int[4];
    __shared__ uint32_t s_flags;
    __shared__ int s_accept;       // decision of the current round
    __shared__ int s_xrem;         // token removed from q after a rejection (-1: none)
    __shared__ float s_qrem;       // its weight e_q as the vector passes compute it
    __shared__ float s_bestv[NWAVES];
    __shared__ int s_besti[NWAVES];

    // Workgroups start in the order y, x.  A sampled sequence costs a workgroup about three
    // times what an argmax sequence costs (two rows, exponentials, k dependent rounds against
    // one row and an argmax), so the sampled sequences are handed out first and the cheap ones
    // fill the end of the launch: sequence number y in dispatch order is the y-th sampled
    // sequence, then the argmax ones in their own order.  Done when B fits the workgroup.
    __shared__ int s_cnt[NWAVES];
    __shared__ int s_seq_of_rank[VT];
    __shared__ float s_T_of_rank[VT];
    // requested now, used after the ranking: the draft-row address needs it (with one tree per
    // sequence the map is that sequence's and can only be read once the sequence is known)
    int qr = p.per_seq ? -1 : p.q_row[row];
    float T = 1.f;
    const bool ranked = p.B > 1 && p.B <= VT;
    if (p.B > 1 && p.B <= 64) {
        // one wavefront ranks up to 64 sequences by itself: one load, one ballot, one barrier
        if (wave == 0) {
            const float Tt = (lane < p.B) ? p.temperature[lane] : 1.f;
            const bool sampled = (lane < p.B) && (Tt != 0.f);
            const unsigned long long m = __ballot(sampled);
            const int total = __popcll(m);
            const int idx_s = __popcll(m & ((1ull << lane) - 1ull));    // sampled sequences before this one
            if (lane < p.B) {
                const int r = sampled ? idx_s : total + (lane - idx_s);
                s_seq_of_rank[r] = lane;
                s_T_of_rank[r] = Tt;
            }
        }
        __syncthreads();
    } else if (ranked) {
        const float Tt = (t < p.B) ? p.temperature[t] : 1.f;
        const bool sampled = (t < p.B) && (Tt != 0.f);
        const unsigned long long m = __ballot(sampled);
        if (lane == 0) s_cnt[wave] = __popcll(m);
        __syncthreads();
        int before = 0, total = 0;
#pragma unroll
        for (int w = 0; w < NWAVES; ++w) {
            const int c = s_cnt[w];
            before += (w < wave) ? c : 0;
            total += c;
        }
        const int idx_s = before + __popcll(m & ((1ull << lane) - 1ull));   // sampled sequences before this one
        if (t < p.B) {
            const int r = sampled ? idx_s : total + (t - idx_s);
            s_seq_of_rank[r] = t;
            s_T_of_rank[r] = Tt;
        }
        __syncthreads();
    }
    if (ranked) {
        // back to wave-uniform values (they come out of LDS): addresses and branches stay scalar,
        // and the temperature does not take a second trip to memory
        b = __builtin_amdgcn_readfirstlane(s_seq_of_rank[blockIdx.y]);
        T = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(s_T_of_rank[blockIdx.y])));
    } else {
        T = p.temperature[b];
    }
    const int32_t *parent = p.parent;
    if (p.per_seq) {
        qr = p.q_row[(size_t)b * (1 + N) + row];
        parent += (size_t)b * N;
    }

    // The two logit rows are requested first; the bookkeeping below (children list, flags)
    // runs while they are in flight.  A row has a draft row iff q_row says so; whether it
    // also has children is checked afterwards (a mismatch is flagged, the row then counts
    // as a leaf and the extra row that was fetched is ignored).
    const size_t rix = (size_t)b * (1 + N) + row;
    const float *zp_row = p.target_logits + rix * (size_t)V;
    const float NaN = __int_as_float(0x7fc00000);
    const bool naive = (p.variant == MCSD_NAIVE);      // the draft row is not needed: candidates are only compared
    const bool have_q = (qr >= 0 && qr < p.P) && (T != 0.f) && !naive;
    const float *zq_row = have_q ? p.draft_logits + ((size_t)b * p.P + qr) * (size_t)V : zp_row;

    // children of this row, ascending node id = sampling order
    if (t < 128) {
        bool f = (t < N) && (parent[t] == row - 1);
        unsigned long long m = __ballot(f);
        if (lane == 0) s_mask[wave] = m;
    }
    if (t == 0) s_flags = 0u;
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
    int k = s_k;
    if (k > 0 && (qr < 0 || qr >= p.P)) {
        // a row with children needs a draft row; a bad map is reported, never dereferenced
        k = 0;
        if (t == 0) atomicOr(&s_flags, (uint32_t)MCSD_FLAG_BAD_TREE);
    }

    if (T == 0.f) {
        // argmax sampling: lowest id on ties; the row is streamed, nothing is kept.  Thread c
        // fetches the token of child c first, so that the comparison after the scan does not
        // wait for memory.
        const int my_tok = (t < k) ? p.cand_tok[(size_t)b * N + s_kids[t]] : -1;
        float bv = -INFINITY;
        int bi = 0x7fffffff;
        stream_row<ITEMS, VT, ALIGNED, true, 16, false>(row_resource(zp_row, V), V, [&](int i, const float4 &z) {
            // A thread meets its elements in ascending token order and the row is padded with
            // -inf past V: a strict comparison keeps the first of equal values, and no bounds
            // check is needed.
            const int e = 4 * (t + VT * i);
            const float v[4] = {z.x, z.y, z.z, z.w};
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (v[c] > bv) { bv = v[c]; bi = e + c; }
        });
        wave_argmax(bv, bi);
        if (lane == 0) { s_bestv[wave] = bv; s_besti[wave] = bi; }
        if (t == 0) s_int[0] = 0x7fffffff;
        __syncthreads();
        bv = s_bestv[0]; bi = s_besti[0];
        for (int w = 1; w < NWAVES; ++w)
            if (s_bestv[w] > bv || (s_bestv[w] == bv && s_besti[w] < bi)) { bv = s_bestv[w]; bi = s_besti[w]; }
        if (bi == 0x7fffffff) bi = 0;
        // the first child (ascending node id) that proposed the argmax is accepted
        if (t < k && my_tok == bi) atomicMin(&s_int[0], t);
        if (t < k && (my_tok < 0 || my_tok >= V)) atomicOr(&s_flags, (uint32_t)MCSD_FLAG_BAD_TOKEN);
        __syncthreads();
        if (t == 0) {
            const int c = s_int[0];
            const int acc = (c < k) ? s_kids[c] : -1;
            p.acc_child[rix] = acc;
            p.endpoint[rix] = acc < 0 ? bi : -1;
            p.flags[rix] = s_flags;
        }
        if (p.ratio && t < k) p.ratio[(size_t)b * N + s_kids[t]] = NaN;
        if (p.residual_out) {
            float *dst = p.residual_out + rix * (size_t)V;
            for (int e = t; e < V; e += VT) dst[e] = (e == bi) ? 1.f : 0.f;
        }
        return;
    }

    // first trip over the draft row (from HBM): its maximum
    float mq = -INFINITY;
    const __amdgpu_buffer_rsrc_t rs_q = row_resource(zq_row, V);
    if (have_q)
        stream_row<ITEMS, VT, ALIGNED, false, 16, false>(rs_q, V, [&](int, const float4 &z) { mq = max3_raw(max3_raw(mq, z.x, z.y), z.z, z.w); });
    // the target row: read exactly once by this workgroup (non-temporal: it does not displace
    // anything in L2), resident from here on.  Requested behind the draft row's first trip, so
    // that its registers are not tied up while that trip runs; it arrives during the bookkeeping
    // below, and the other workgroup of the compute unit computes meanwhile.
    float4 a[ITEMS];
    {
        const __amdgpu_buffer_rsrc_t rs_p = row_resource(zp_row, V);
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) a[i] = load_row_piece<VT, ALIGNED, true>(rs_p, i, V, t);
    }

    // Thread c follows candidate c: its token, its uniform and the two logits of that token are
    // requested now, so that the first accept decision does not wait for three dependent trips
    // to memory after the exponentials.
    int my_tok = -1;
    float my_u = 0.f, my_zp = 0.f, my_zq = 0.f;
    if (k > 0 && !naive && t < k) {
        const int node = s_kids[t];
        my_tok = p.cand_tok[(size_t)b * N + node];
        my_u = p.u_accept[(size_t)b * N + node];
        if (my_tok >= 0 && my_tok < V) {
            my_zp = zp_row[my_tok];
            my_zq = zq_row[my_tok];
        }
    }
    const float invT = 1.0f / T;
    const float c2 = invT * LOG2E_F;
    float mp = row_max<ITEMS>(a);
    block_max2<NWAVES>(mp, mq, s_redf, s_redf2);
    double A = row_exp<ITEMS>(a, mp, c2);                 // a = e_p, A = Z_p
    double Zq0 = 0.0;
    if (k > 0 && !naive)                                   // second trip over the draft row: sum of e_q
        stream_row<ITEMS, VT, ALIGNED, false, PASS_CHUNK, PASS_DOUBLE>(rs_q, V, [&](int, const float4 &z) { Zq0 += sum4(exp_weights(z, mq, c2)); });
    block_sum2<NWAVES>(A, Zq0, s_red, s_red2);
    if (!(A > 0.0) || !isfinite(A) || (k > 0 && !naive && (!(Zq0 > 0.0) || !isfinite(Zq0)))) {
        if (t == 0) atomicOr(&s_flags, (uint32_t)MCSD_FLAG_NONFINITE);
    }

    int accepted = -1;
    if (k > 0 && !naive) {
        // fp64 track of the candidate tokens: thread c follows candidate c
        double my_a = 0.0, my_q = 0.0;
        float my_q32 = 0.f;                 // e_q of the token with the rounding of the vector passes
        if (t < k && my_tok >= 0 && my_tok < V) {
            // same constants as the vector pass (float c2), evaluated exactly
            my_a = exp2_neg(((double)my_zp - (double)mp) * (double)c2);
            my_q = exp2_neg(((double)my_zq - (double)mq) * (double)c2);
            my_q32 = __builtin_amdgcn_exp2f((my_zq - mq) * c2);
        }
        // Z_q: mass of the draft tokens not yet removed.  A removal takes away exactly the fp32
        // weight that the sum over the row contained for that token (the same instructions on
        // the same logit give the same bits), so the difference keeps its relative accuracy
        // even when most of the mass has been removed.
        double Zq = Zq0;

        for (int i = 0; i < k; ++i) {
            if (t == i) {
                const VerifyParams pl = reload_params();
                double ratio;
                uint32_t fl = 0u;
                const bool valid = (my_tok >= 0 && my_tok < V);
                if (!valid) {
                    ratio = 0.0;
                    fl |= MCSD_FLAG_BAD_TOKEN;
                } else if (my_q > 0.0) {
                    ratio = (my_a * Zq) / (A * my_q);
                    if (!(ratio < 1.0)) ratio = 1.0;
                } else {
                    ratio = my_a > 0.0 ? 1.0 : 0.0;
                    fl |= MCSD_FLAG_ZERO_DRAFT_PROB;
                }
                const double u = (double)my_u;
                // (a token of probability zero - a duplicate of a rejected one, Sec. 3.2 - is never
                // accepted, also not by a uniform of exactly 0 from outside the open interval)
                const bool acc = (ratio > 0.0) && (u <= ratio);
                if (fabs(u - ratio) < (double)pl.eps) fl |= MCSD_FLAG_NEAR_TIE_ACCEPT;
                if (fl) atomicOr(&s_flags, fl);
                if (pl.ratio) pl.ratio[(size_t)b * N + s_kids[i]] = (float)ratio;
                s_accept = acc ? 1 : 0;
                const bool remove = (!acc) && valid && (pl.variant == MCSD_WITHOUT_REPLACEMENT);
                s_xrem = remove ? my_tok : -1;
                s_qrem = remove ? my_q32 : 0.f;
            }
            __syncthreads();
            if (s_accept) {
                accepted = i;
                break;
            }
            // rejected: a := max(0, a - beta e_q) with beta = A / Z_q in fp64, applied as a
            // two-term float product so that no common rounding of beta biases the sum
            const double beta = (Zq > 0.0) ? A / Zq : 0.0;   // nothing left in q: the residual is p itself
            const int xrem = s_xrem;
            const double Zq_new = Zq - (double)s_qrem;
            const float bh = (float)beta;
            const float bl = (float)(beta - (double)bh);
            double part = 0.0;
            // one more trip over the draft row for e_q
            stream_row<ITEMS, VT, ALIGNED, false, PASS_CHUNK, PASS_DOUBLE>(rs_q, V, [&](int j, const float4 &z) {
                const float4 e = exp_weights(z, mq, c2);
                a[j].x = fmaxf(0.f, fmaf(-bl, e.x, fmaf(-bh, e.x, a[j].x)));
                a[j].y = fmaxf(0.f, fmaf(-bl, e.y, fmaf(-bh, e.y, a[j].y)));
                a[j].z = fmaxf(0.f, fmaf(-bl, e.z, fmaf(-bh, e.z, a[j].z)));
                a[j].w = fmaxf(0.f, fmaf(-bl, e.w, fmaf(-bh, e.w, a[j].w)));
                part += sum4(a[j]);
            });
            const double my_a_new = fmax(0.0, my_a - beta * my_q);
            if (t < k && xrem >= 0 && my_tok == xrem) { my_q = 0.0; my_q32 = 0.f; }
            const double A_new = block_sum<NWAVES>(part, s_red);     // barriers inside also order the reuse of s_accept / s_xrem / s_qrem
            Zq = Zq_new;
            if (A_new > 0.0) {
                A = A_new;
                my_a = my_a_new;
            } else {
                // max(0, p - q) vanished everywhere, which a rejection excludes in exact arithmetic
                // (it needs p = q) and rounding or a bad candidate can produce: p stays as it
                // was.  With every a(x) <= beta e_q(x) and equal sums, the old a is beta e_q.
                if (t == 0) atomicOr(&s_flags, (uint32_t)MCSD_FLAG_ZERO_RESIDUAL);
                stream_row<ITEMS, VT, ALIGNED, false, PASS_CHUNK, PASS_DOUBLE>(rs_q, V, [&](int j, const float4 &z) {
                    const float4 e = exp_weights(z, mq, c2);
                    a[j] = make_float4(fmaf(bl, e.x, bh * e.x), fmaf(bl, e.y, bh * e.y), fmaf(bl, e.z, bh * e.z), fmaf(bl, e.w, bh * e.w));
                });
            }
        }
        // candidates after the accepted one were never tested
        const VerifyParams pl = reload_params();
        if (pl.ratio && accepted >= 0 && t > accepted && t < k) pl.ratio[(size_t)b * N + s_kids[t]] = NaN;
    }

    const VerifyParams pe = reload_params();
    int endpoint = -1;
    if (accepted < 0) {
        const double u = (double)pe.u_endpoint[rix];
        endpoint = inverse_cdf<ITEMS, VT>(a, A, u, (double)pe.eps, s_red, s_seg, s_int, &s_flags);
        if (endpoint < 0 || endpoint >= V) endpoint = V - 1;
    }
    if (naive && k > 0) {
        // multi-candidate naive sampling (the comparison rule of the ablation, Sec. 4.5): the
        // token just drawn from p is kept; a candidate equal to it is accepted, the first such
        if (t == 0) {
            int acc = -1;
            uint32_t fl = 0u;
            for (int i = 0; i < k; ++i) {
                const int tok = pe.cand_tok[(size_t)b * N + s_kids[i]];
                if (tok < 0 || tok >= V) fl |= MCSD_FLAG_BAD_TOKEN;
                else if (acc < 0 && tok == endpoint) acc = i;
            }
            if (fl) atomicOr(&s_flags, fl);
            s_accept = acc;
        }
        if (pe.ratio && t < k) pe.ratio[(size_t)b * N + s_kids[t]] = NaN;
        __syncthreads();
        accepted = s_accept;
        if (accepted >= 0) endpoint = -1;
    }
    if (pe.residual_out) {
        const float inv = (A > 0.0) ? (float)(1.0 / A) : 0.f;
        store_residual<ITEMS, VT, ALIGNED>(pe.residual_out + rix * (size_t)V, V, a, inv);
    }
    __syncthreads();
    if (t == 0) {
        pe.acc_child[rix] = accepted >= 0 ? s_kids[accepted] : -1;
        pe.endpoint[rix] = endpoint;
        pe.flags[rix] = s_flags;
    }
}

// ---------------------------------------------------------------- both rows resident
// Vocabularies up to 32768: one workgroup per tree row, both logit rows of the row in registers
// for all rounds (1024 threads up to 16384 tokens, 512 threads with twice the registers beyond).
template <int ITEMS, int VT, bool ALIGNED>
__global__ __launch_bounds__(VT) void verify_rows_kernel(VerifyParams p)
{
    constexpr int NWAVES = VT / 64;
    const int row = blockIdx.x;
    int b = blockIdx.y;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int N = p.N, V = p.V;

    __shared__ double s_red[NWAVES];
    __shared__ double s_red2[NWAVES];
    __shared__ double s_seg[4 * NWAVES * ITEMS + ITEMS];
    __shared__ float s_redf[NWAVES];
    __shared__ float s_redf2[NWAVES];
    __shared__ unsigned long long s_mask[2];
    __shared__ int s_kids[MCSD_MAX_NODES];
    __shared__ int s_k;
    __shared__ int s_int[4];
    __shared__ uint32_t s_flags;
    __shared__ int s_accept;       // decision of the current round
    __shared__ int s_xrem;         // token removed from q after a rejection (-1: none)
    __shared__ float s_bestv[NWAVES];
    __shared__ int s_besti[NWAVES];

    // Workgroups start in the order y, x.  A sampled sequence costs a workgroup about three
    // times what an argmax sequence costs (two rows, exponentials, k dependent rounds against
    // one row and an argmax), so the sampled sequences are handed out first and the cheap ones
    // fill the end of the launch: sequence number y in dispatch order is the y-th sampled
    // sequence, then the argmax ones in their own order.  Done when B fits the workgroup.
    __shared__ int s_cnt[NWAVES];
    __shared__ int s_seq_of_rank[VT];
    __shared__ float s_T_of_rank[VT];
    // requested now, used after the ranking: the draft-row address needs it (with one tree per
    // sequence the map is that sequence's and can only be read once the sequence is known)
    int qr = p.per_seq ? -1 : p.q_row[row];
    float T = 1.f;
    const bool ranked = p.B > 1 && p.B <= VT;
    if (p.B > 1 && p.B <= 64) {
        // one wavefront ranks up to 64 sequences by itself: one load, one ballot, one barrier
        if (wave == 0) {
            const float Tt = (lane < p.B) ? p.temperature[lane] : 1.f;
            const bool sampled = (lane < p.B) && (Tt != 0.f);
            const unsigned long long m = __ballot(sampled);
            const int total = __popcll(m);
            const int idx_s = __popcll(m & ((1ull << lane) - 1ull));    // sampled sequences before this one
            if (lane < p.B) {
                const int r = sampled ? idx_s : total + (lane - idx_s);
                s_seq_of_rank[r] = lane;
                s_T_of_rank[r] = Tt;
            }
        }
        __syncthreads();
    } else if (ranked) {
        const float Tt = (t < p.B) ? p.temperature[t] : 1.f;
        const bool sampled = (t < p.B) && (Tt != 0.f);
        const unsigned long long m = __ballot(sampled);
        if (lane == 0) s_cnt[wave] = __popcll(m);
        __syncthreads();
        int before = 0, total = 0;
#pragma unroll
        for (int w = 0; w < NWAVES; ++w) {
            const int c = s_cnt[w];
            before += (w < wave) ? c : 0;
            total += c;
        }
        const int idx_s = before + __popcll(m & ((1ull << lane) - 1ull));   // sampled sequences before this one
        if (t < p.B) {
            const int r = sampled ? idx_s : total + (t - idx_s);
            s_seq_of_rank[r] = t;
            s_T_of_rank[r] = Tt;
        }
        __syncthreads();
    }
    if (ranked) {
        // back to wave-uniform values (they come out of LDS): addresses and branches stay scalar,
        // and the temperature does not take a second trip to memory
        b = __builtin_amdgcn_readfirstlane(s_seq_of_rank[blockIdx.y]);
        T = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(s_T_of_rank[blockIdx.y])));
    } else {
        T = p.temperature[b];
    }
    const int32_t *parent = p.parent;
    if (p.per_seq) {
        qr = p.q_row[(size_t)b * (1 + N) + row];
        parent += (size_t)b * N;
    }

    // The two logit rows are requested first; the bookkeeping below (children list, flags)
    // runs while they are in flight.  A row has a draft row iff q_row says so; whether it
    // also has children is checked afterwards (a mismatch is flagged, the row then counts
    // as a leaf and the extra row that was fetched is ignored).
    const size_t rix = (size_t)b * (1 + N) + row;
    const float *zp_row = p.target_logits + rix * (size_t)V;
    const float NaN = __int_as_float(0x7fc00000);
    float4 a[ITEMS];
    {
        const __amdgpu_buffer_rsrc_t rs_p = row_resource(zp_row, V);
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) a[i] = load_row_piece<VT, ALIGNED, true>(rs_p, i, V, t);
    }
    const bool naive = (p.variant == MCSD_NAIVE);      // the draft row is not needed: candidates are only compared
    const bool have_q = (qr >= 0 && qr < p.P) && (T != 0.f) && !naive;
    const float *zq_row = have_q ? p.draft_logits + ((size_t)b * p.P + qr) * (size_t)V : zp_row;
    float4 eq[ITEMS];
    if (have_q) {
        const __amdgpu_buffer_rsrc_t rs_q = row_resource(zq_row, V);
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) eq[i] = load_row_piece<VT, ALIGNED, true>(rs_q, i, V, t);
    } else {
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) eq[i] = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
    }

    // children of this row, ascending node id = sampling order
    if (t < 128) {
        bool f = (t < N) && (parent[t] == row - 1);
        unsigned long long m = __ballot(f);
        if (lane == 0) s_mask[wave] = m;
    }
    if (t == 0) s_flags = 0u;
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
    int k = s_k;
    if (k > 0 && (qr < 0 || qr >= p.P)) {
        // a row with children needs a draft row; a bad map is reported, never dereferenced
        k = 0;
        if (t == 0) atomicOr(&s_flags, (uint32_t)MCSD_FLAG_BAD_TREE);
    }

    if (T == 0.f) {
        // argmax sampling: lowest id on ties.  Thread c fetches the token of child c now, so that
        // the comparison after the scan does not wait for memory.
        const int my_tok = (t < k) ? p.cand_tok[(size_t)b * N + s_kids[t]] : -1;
        float bv = -INFINITY;
        int bi = 0x7fffffff;
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            // A thread meets its elements in ascending token order and the row was padded with
            // -inf past V when it was loaded: a strict comparison keeps the first of equal
            // values, and no bounds check is needed.
            const int e = 4 * (t + VT * i);
            const float v[4] = {a[i].x, a[i].y, a[i].z, a[i].w};
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (v[c] > bv) { bv = v[c]; bi = e + c; }
        }
        wave_argmax(bv, bi);
        if (lane == 0) { s_bestv[wave] = bv; s_besti[wave] = bi; }
        if (t == 0) s_int[0] = 0x7fffffff;
        __syncthreads();
        bv = s_bestv[0]; bi = s_besti[0];
        for (int w = 1; w < NWAVES; ++w)
            if (s_bestv[w] > bv || (s_bestv[w] == bv && s_besti[w] < bi)) { bv = s_bestv[w]; bi = s_besti[w]; }
        if (bi == 0x7fffffff) bi = 0;
        // the first child (ascending node id) that proposed the argmax is accepted
        if (t < k && my_tok == bi) atomicMin(&s_int[0], t);
        if (t < k && (my_tok < 0 || my_tok >= V)) atomicOr(&s_flags, (uint32_t)MCSD_FLAG_BAD_TOKEN);
        __syncthreads();
        if (t == 0) {
            const int c = s_int[0];
            const int acc = (c < k) ? s_kids[c] : -1;
            p.acc_child[rix] = acc;
            p.endpoint[rix] = acc < 0 ? bi : -1;
            p.flags[rix] = s_flags;
        }
        if (p.ratio && t < k) p.ratio[(size_t)b * N + s_kids[t]] = NaN;
        if (p.residual_out) {
            float *dst = p.residual_out + rix * (size_t)V;
            for (int e = t; e < V; e += VT) dst[e] = (e == bi) ? 1.f : 0.f;
        }
        return;
    }

    // Thread c follows candidate c: its token, its uniform and the two logits of that token are
    // requested now, so that the first accept decision does not wait for three dependent trips
    // to memory after the exponentials.
    int my_tok = -1;
    float my_u = 0.f, my_zp = 0.f, my_zq = 0.f;
    if (k > 0 && !naive && t < k) {
        const int node = s_kids[t];
        my_tok = p.cand_tok[(size_t)b * N + node];
        my_u = p.u_accept[(size_t)b * N + node];
        if (my_tok >= 0 && my_tok < V) {
            my_zp = zp_row[my_tok];
            my_zq = zq_row[my_tok];
        }
    }
    const float invT = 1.0f / T;
    const float c2 = invT * LOG2E_F;
    float mp = row_max<ITEMS>(a), mq = row_max<ITEMS>(eq);
    block_max2<NWAVES>(mp, mq, s_redf, s_redf2);
    double A = row_exp<ITEMS>(a, mp, c2);                 // a = e_p, A = Z_p
    double Zq0 = (k > 0 && !naive) ? row_exp<ITEMS>(eq, mq, c2) : 0.0;
    block_sum2<NWAVES>(A, Zq0, s_red, s_red2);
    if (!(A > 0.0) || !isfinite(A) || (k > 0 && !naive && (!(Zq0 > 0.0) || !isfinite(Zq0)))) {
        if (t == 0) atomicOr(&s_flags, (uint32_t)MCSD_FLAG_NONFINITE);
    }

    int accepted = -1;
    if (k > 0 && !naive) {
        // fp64 track of the candidate tokens: thread c follows candidate c
        double my_a = 0.0, my_q = 0.0;
        if (t < k && my_tok >= 0 && my_tok < V) {
            // same constants as the vector pass (float c2), evaluated exactly
            my_a = exp2_neg(((double)my_zp - (double)mp) * (double)c2);
            my_q = exp2_neg(((double)my_zq - (double)mq) * (double)c2);
        }
        // Z_q: mass of the draft tokens not yet removed.  After a removal it is summed
        // again over the resident row rather than updated by subtraction, so that it
        // keeps its relative accuracy when most of the mass has been removed.
        double Zq = Zq0;

        for (int i = 0; i < k; ++i) {
            if (t == i) {
                double ratio;
                uint32_t fl = 0u;
                const bool valid = (my_tok >= 0 && my_tok < V);
                if (!valid) {
                    ratio = 0.0;
                    fl |= MCSD_FLAG_BAD_TOKEN;
                } else if (my_q > 0.0) {
                    ratio = (my_a * Zq) / (A * my_q);
                    if (!(ratio < 1.0)) ratio = 1.0;
                } else {
                    ratio = my_a > 0.0 ? 1.0 : 0.0;
                    fl |= MCSD_FLAG_ZERO_DRAFT_PROB;
                }
                const double u = (double)my_u;
                // (a token of probability zero - a duplicate of a rejected one, Sec. 3.2 - is never
                // accepted, also not by a uniform of exactly 0 from outside the open interval)
                const bool acc = (ratio > 0.0) && (u <= ratio);
                if (fabs(u - ratio) < (double)p.eps) fl |= MCSD_FLAG_NEAR_TIE_ACCEPT;
                if (fl) atomicOr(&s_flags, fl);
                if (p.ratio) p.ratio[(size_t)b * N + s_kids[i]] = (float)ratio;
                s_accept = acc ? 1 : 0;
                const bool remove = (!acc) && valid && (p.variant == MCSD_WITHOUT_REPLACEMENT);
                s_xrem = remove ? my_tok : -1;
            }
            __syncthreads();
            if (s_accept) {
                accepted = i;
                break;
            }
            // rejected: a := max(0, a - beta e_q) with beta = A / Z_q in fp64, applied as a
            // two-term float product so that no common rounding of beta biases the sum
            const double beta = (Zq > 0.0) ? A / Zq : 0.0;   // nothing left in q: the residual is p itself
            const int xrem = s_xrem;
            const float bh = (float)beta;
            const float bl = (float)(beta - (double)bh);
            double part = 0.0, partq = 0.0;
#pragma unroll
            for (int j = 0; j < ITEMS; ++j) {
                a[j].x = fmaxf(0.f, fmaf(-bl, eq[j].x, fmaf(-bh, eq[j].x, a[j].x)));
                a[j].y = fmaxf(0.f, fmaf(-bl, eq[j].y, fmaf(-bh, eq[j].y, a[j].y)));
                a[j].z = fmaxf(0.f, fmaf(-bl, eq[j].z, fmaf(-bh, eq[j].z, a[j].z)));
                a[j].w = fmaxf(0.f, fmaf(-bl, eq[j].w, fmaf(-bh, eq[j].w, a[j].w)));
                part += sum4(a[j]);
            }
            const double my_a_new = fmax(0.0, my_a - beta * my_q);
            if (t < k && xrem >= 0 && my_tok == xrem) my_q = 0.0;
            double A_new;
            if (xrem >= 0) {
                const int q4 = xrem >> 2;                 // float4 index of the removed token
                if ((q4 & (VT - 1)) == t) {
                    const int j = q4 / VT, c = xrem & 3;
#pragma unroll
                    for (int jj = 0; jj < ITEMS; ++jj)
                        if (jj == j) {
                            if (c == 0) eq[jj].x = 0.f;
                            if (c == 1) eq[jj].y = 0.f;
                            if (c == 2) eq[jj].z = 0.f;
                            if (c == 3) eq[jj].w = 0.f;
                        }
                }
#pragma unroll
                for (int j = 0; j < ITEMS; ++j)
                    partq += sum4(eq[j]);
                block_sum2<NWAVES>(part, partq, s_red, s_red2);   // barriers inside also order the reuse of s_accept / s_xrem
                A_new = part;
                Zq = partq;
            } else {
                A_new = block_sum<NWAVES>(part, s_red);
            }
            if (A_new > 0.0) {
                A = A_new;
                my_a = my_a_new;
            } else {
                // max(0, p - q) vanished everywhere, which a rejection excludes in exact arithmetic
                // (it needs p = q) and rounding or a bad candidate can produce: p stays as it
                // was.  With every a(x) <= beta e_q(x) and equal sums, the old a is beta e_q.
                if (t == 0) atomicOr(&s_flags, (uint32_t)MCSD_FLAG_ZERO_RESIDUAL);
#pragma unroll
                for (int j = 0; j < ITEMS; ++j) {
                    a[j].x = fmaf(bl, eq[j].x, bh * eq[j].x);
                    a[j].y = fmaf(bl, eq[j].y, bh * eq[j].y);
                    a[j].z = fmaf(bl, eq[j].z, bh * eq[j].z);
                    a[j].w = fmaf(bl, eq[j].w, bh * eq[j].w);
                }
            }
        }
        // candidates after the accepted one were never tested
        if (p.ratio && accepted >= 0 && t > accepted && t < k) p.ratio[(size_t)b * N + s_kids[t]] = NaN;
    }

    int endpoint = -1;
    if (accepted < 0) {
        const double u = (double)p.u_endpoint[rix];
        endpoint = inverse_cdf<ITEMS, VT>(a, A, u, (double)p.eps, s_red, s_seg, s_int, &s_flags);
        if (endpoint < 0 || endpoint >= V) endpoint = V - 1;
    }
    if (naive && k > 0) {
        // multi-candidate naive sampling (the comparison rule of the ablation, Sec. 4.5): the
        // token just drawn from p is kept; a candidate equal to it is accepted, the first such
        if (t == 0) {
            int acc = -1;
            uint32_t fl = 0u;
            for (int i = 0; i < k; ++i) {
                const int tok = p.cand_tok[(size_t)b * N + s_kids[i]];
                if (tok < 0 || tok >= V) fl |= MCSD_FLAG_BAD_TOKEN;
                else if (acc < 0 && tok == endpoint) acc = i;
            }
            if (fl) atomicOr(&s_flags, fl);
            s_accept = acc;
        }
        if (p.ratio && t < k) p.ratio[(size_t)b * N + s_kids[t]] = NaN;
        __syncthreads();
        accepted = s_accept;
        if (accepted >= 0) endpoint = -1;
    }
    if (p.residual_out) {
        const float inv = (A > 0.0) ? (float)(1.0 / A) : 0.f;
        store_residual<ITEMS, VT, ALIGNED>(p.residual_out + rix * (size_t)V, V, a, inv);
    }
    __syncthreads();
    if (t == 0) {
        p.acc_child[rix] = accepted >= 0 ? s_kids[accepted] : -1;
        p.endpoint[rix] = endpoint;
        p.flags[rix] = s_flags;
    }
}

__global__ void walk_kernel(WalkParams w)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < w.B) walk_sequence(w, b);
}

template <int ITEMS, int VT>
void launch_rows(const VerifyParams &p, hipStream_t stream)
{
    dim3 grid(1 + p.N, p.B), block(VT);
    if (p.V % 4 == 0)
        launch_kernel(K_VERIFY_ROWS, verify_rows_kernel<ITEMS, VT, true>, grid, block, stream, p);
    else
        launch_kernel(K_VERIFY_ROWS, verify_rows_kernel<ITEMS, VT, false>, grid, block, stream, p);
}

template <int ITEMS, int VT>
void launch_rows_stream(const VerifyParams &p, hipStream_t stream)
{
    dim3 grid(1 + p.N, p.B), block(VT);
    if (p.V % 4 == 0)
        launch_kernel(K_VERIFY_ROWS, verify_rows_stream_kernel<ITEMS, VT, true>, grid, block, stream, p);
    else
        launch_kernel(K_VERIFY_ROWS, verify_rows_stream_kernel<ITEMS, VT, false>, grid, block, stream, p);
}

}  // namespace

WalkParams make_walk_params(const mcsd_verify_desc &d, const mcsd_verify_bufs &b)
{
    WalkParams w;
    w.B = d.B; w.N = d.N; w.gamma_max = d.gamma_max; w.flags = b.flags;
    w.acc_child = b.acc_child; w.endpoint = b.endpoint; w.cand_tok = b.cand_tok;
    w.n_accepted = b.n_accepted; w.accepted_path = b.accepted_path; w.out_tokens = b.out_tokens;
    return w;
}

int32_t launch_verify(const mcsd_verify_desc &d, const mcsd_verify_bufs &b, hipStream_t stream, bool with_walk)
{
    VerifyParams p;
    p.B = d.B; p.N = d.N; p.V = d.V; p.P = d.P; p.variant = d.variant; p.gamma_max = d.gamma_max;
    p.eps = d.near_tie_eps; p.per_seq = d.parent_per_seq;
    p.target_logits = b.target_logits; p.draft_logits = b.draft_logits;
    p.q_row = b.q_row; p.parent = b.parent; p.cand_tok = b.cand_tok;
    p.u_accept = b.u_accept; p.u_endpoint = b.u_endpoint; p.temperature = b.temperature;
    p.n_accepted = b.n_accepted; p.accepted_path = b.accepted_path; p.out_tokens = b.out_tokens;
    p.acc_child = b.acc_child; p.endpoint = b.endpoint; p.ratio = b.ratio; p.flags = b.flags;
    p.residual_out = b.residual_out;

    // Up to 32768 tokens both logit rows of a node stay in the registers of one workgroup (1024
    // threads up to 16384 tokens, 512 threads with twice the registers each beyond that); larger
    // vocabularies keep the target row only and stream the draft row.
    const int items1024 = (d.V + 4095) / 4096;
    if (items1024 <= 1) launch_rows<1, 1024>(p, stream);
    else if (items1024 <= 2) launch_rows<2, 1024>(p, stream);
    else if (items1024 <= 4) launch_rows<4, 1024>(p, stream);
    else if (items1024 <= 8) launch_rows<16, 512>(p, stream);
    else launch_rows_stream<32, 512>(p, stream);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_error("verify_rows launch failed: %s", hipGetErrorString(e));
        return MCSD_E_HIP;
    }
    if (!with_walk) return MCSD_OK;
    launch_kernel(K_WALK, walk_kernel, dim3((d.B + 63) / 64), dim3(64), stream, make_walk_params(d, b));
    e = hipGetLastError();
    if (e != hipSuccess) {
        set_error("walk launch failed: %s", hipGetErrorString(e));
        return MCSD_E_HIP;
    }
    return MCSD_OK;
}

}  // namespace mcsd
