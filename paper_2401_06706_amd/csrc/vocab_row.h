// Device helpers for kernels in which one workgroup holds one vocabulary row (float4 x ITEMS
// per thread, VT threads): wavefront / workgroup reductions, the row load, the exponential
// pass and the inverse-CDF search.  Shared by the verification and the draft-sampling kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include <type_traits>

#include "mcsd.h"

namespace mcsd {
namespace vocab {

// Wavefront reductions on the DPP cross-lane paths (no LDS round trip).  The result is
// complete in lane 63 only: quad swaps, half-row and row mirrors give every lane its row's
// total, then row_bcast15 / row_bcast31 fold the four rows of 16 lanes into the last one.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_f(float old, float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(old), __float_as_int(v), CTRL, ROW_MASK, 0xf, false));
}

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_d(double old, double v)
{
    const long long o = __double_as_longlong(old), x = __double_as_longlong(v);
    const int lo = __builtin_amdgcn_update_dpp((int)o, (int)x, CTRL, ROW_MASK, 0xf, false);
    const int hi = __builtin_amdgcn_update_dpp((int)(o >> 32), (int)(x >> 32), CTRL, ROW_MASK, 0xf, false);
    return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}

constexpr int DPP_QUAD_1032 = 0xB1, DPP_QUAD_2301 = 0x4E, DPP_ROW_HALF_MIRROR = 0x141, DPP_ROW_MIRROR = 0x140,
              DPP_ROW_BCAST15 = 0x142, DPP_ROW_BCAST31 = 0x143,
              DPP_ROW_SHR1 = 0x111, DPP_ROW_SHR2 = 0x112, DPP_ROW_SHR4 = 0x114, DPP_ROW_SHR8 = 0x118;

__device__ __forceinline__ float wave_max(float v)      // valid in lane 63
{
    v = fmaxf(v, dpp_f<DPP_QUAD_1032, 0xf>(v, v));
    v = fmaxf(v, dpp_f<DPP_QUAD_2301, 0xf>(v, v));
    v = fmaxf(v, dpp_f<DPP_ROW_HALF_MIRROR, 0xf>(v, v));
    v = fmaxf(v, dpp_f<DPP_ROW_MIRROR, 0xf>(v, v));
    v = fmaxf(v, dpp_f<DPP_ROW_BCAST15, 0xa>(v, v));
    v = fmaxf(v, dpp_f<DPP_ROW_BCAST31, 0xc>(v, v));
    return v;
}

__device__ __forceinline__ int wave_min(int v)           // valid in lane 63
{
    v = min(v, __builtin_amdgcn_update_dpp(v, v, DPP_QUAD_1032, 0xf, 0xf, false));
    v = min(v, __builtin_amdgcn_update_dpp(v, v, DPP_QUAD_2301, 0xf, 0xf, false));
    v = min(v, __builtin_amdgcn_update_dpp(v, v, DPP_ROW_HALF_MIRROR, 0xf, 0xf, false));
    v = min(v, __builtin_amdgcn_update_dpp(v, v, DPP_ROW_MIRROR, 0xf, 0xf, false));
    v = min(v, __builtin_amdgcn_update_dpp(v, v, DPP_ROW_BCAST15, 0xa, 0xf, false));
    v = min(v, __builtin_amdgcn_update_dpp(v, v, DPP_ROW_BCAST31, 0xc, 0xf, false));
    return v;
}

// Largest value of the wavefront and the lowest index among the lanes that hold it, in every
// lane: two DPP reductions and two lane reads instead of six rounds of cross-lane shuffles.
__device__ __forceinline__ void wave_argmax(float &bv, int &bi)
{
    const float m = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(wave_max(bv)), 63));
    const int i = wave_min(bv == m ? bi : 0x7fffffff);
    bv = m;
    bi = __builtin_amdgcn_readlane(i, 63);
}

__device__ __forceinline__ double wave_sum(double v)    // valid in lane 63
{
    v += dpp_d<DPP_QUAD_1032, 0xf>(0.0, v);
    v += dpp_d<DPP_QUAD_2301, 0xf>(0.0, v);
    v += dpp_d<DPP_ROW_HALF_MIRROR, 0xf>(0.0, v);
    v += dpp_d<DPP_ROW_MIRROR, 0xf>(0.0, v);
    v += dpp_d<DPP_ROW_BCAST15, 0xa>(0.0, v);
    v += dpp_d<DPP_ROW_BCAST31, 0xc>(0.0, v);
    return v;
}

// Inclusive running sum over the lanes of the wavefront: shifts inside the rows of 16 lanes
// (a lane without a source adds zero), then the totals of the rows before it.
__device__ __forceinline__ double wave_scan_inclusive(double v)
{
    v += dpp_d<DPP_ROW_SHR1, 0xf>(0.0, v);
    v += dpp_d<DPP_ROW_SHR2, 0xf>(0.0, v);
    v += dpp_d<DPP_ROW_SHR4, 0xf>(0.0, v);
    v += dpp_d<DPP_ROW_SHR8, 0xf>(0.0, v);
    v += dpp_d<DPP_ROW_BCAST15, 0xa>(0.0, v);
    v += dpp_d<DPP_ROW_BCAST31, 0xc>(0.0, v);
    return v;
}

// ITEMS values per lane -> for every row of 16 lanes, the 16-lane total of each of the ITEMS
// values, spread over the lanes of that row: lane l ends up with the total of value number
// `which`.  Each of the first log2(ITEMS) steps halves the values a lane carries: the partner
// (whose lane number differs in the step's bit) gets the half this lane gives up, and this lane
// adds the partner's copy of the half it keeps.  15 exchanges for 16 values instead of 16 x 4.
template <int ITEMS>
__device__ __forceinline__ double row_totals_scattered(double (&x)[ITEMS], int lane, int &which)
{
    static_assert(ITEMS == 1 || ITEMS == 2 || ITEMS == 4 || ITEMS == 8 || ITEMS == 16, "power of two up to 16");
    which = 0;
    auto step = [&](auto ctrl_c, auto n_c, int bit) __attribute__((always_inline)) {
        constexpr int CTRL = decltype(ctrl_c)::value;
        constexpr int N = decltype(n_c)::value;          // values carried before this step
        if constexpr (N > 1) {
            const bool keep_hi = (lane >> bit) & 1;
#pragma unroll
            for (int j = 0; j < N / 2; ++j) {
                const double mine = keep_hi ? x[j + N / 2] : x[j];
                const double give = keep_hi ? x[j] : x[j + N / 2];
                x[j] = mine + dpp_d<CTRL, 0xf>(0.0, give);
            }
            if (keep_hi) which += N / 2;
        } else {
            x[0] += dpp_d<CTRL, 0xf>(0.0, x[0]);
        }
    };
    // Widest exchange first: the row mirror (lane i <-> 15 - i) flips bit 3, and every later
    // exchange (mirror inside 8 lanes, lanes 2 apart, neighbours) leaves the bits of the earlier
    // steps alone, so the two partners of a step always carry the same subset of the values.
    step(std::integral_constant<int, DPP_ROW_MIRROR>(), std::integral_constant<int, ITEMS>(), 3);
    step(std::integral_constant<int, DPP_ROW_HALF_MIRROR>(), std::integral_constant<int, (ITEMS > 1 ? ITEMS / 2 : 1)>(), 2);
    step(std::integral_constant<int, DPP_QUAD_2301>(), std::integral_constant<int, (ITEMS > 2 ? ITEMS / 4 : 1)>(), 1);
    step(std::integral_constant<int, DPP_QUAD_1032>(), std::integral_constant<int, (ITEMS > 4 ? ITEMS / 8 : 1)>(), 0);
    return x[0];
}

// Every thread returns the same value (fixed summation order over the waves).
template <int NWAVES>
__device__ __forceinline__ double block_sum(double v, double *s_red)
{
    v = wave_sum(v);
    if ((threadIdx.x & 63) == 63) s_red[threadIdx.x >> 6] = v;
    __syncthreads();
    double r = 0.0;
#pragma unroll
    for (int w = 0; w < NWAVES; ++w) r += s_red[w];
    __syncthreads();
    return r;
}

// Two sums in one pass (same barriers): a -> first, b -> second.
template <int NWAVES>
__device__ __forceinline__ void block_sum2(double &a, double &b, double *s_red, double *s_red2)
{
    a = wave_sum(a);
    b = wave_sum(b);
    if ((threadIdx.x & 63) == 63) { s_red[threadIdx.x >> 6] = a; s_red2[threadIdx.x >> 6] = b; }
    __syncthreads();
    double ra = 0.0, rb = 0.0;
#pragma unroll
    for (int w = 0; w < NWAVES; ++w) { ra += s_red[w]; rb += s_red2[w]; }
    __syncthreads();
    a = ra;
    b = rb;
}

template <int NWAVES>
__device__ __forceinline__ float block_max(float v, float *s_red)
{
    v = wave_max(v);
    if ((threadIdx.x & 63) == 63) s_red[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = s_red[0];
#pragma unroll
    for (int w = 1; w < NWAVES; ++w) r = fmaxf(r, s_red[w]);
    __syncthreads();
    return r;
}

// Two maxima in one pass.
template <int NWAVES>
__device__ __forceinline__ void block_max2(float &a, float &b, float *s_red, float *s_red2)
{
    a = wave_max(a);
    b = wave_max(b);
    if ((threadIdx.x & 63) == 63) { s_red[threadIdx.x >> 6] = a; s_red2[threadIdx.x >> 6] = b; }
    __syncthreads();
    float ra = s_red[0], rb = s_red2[0];
#pragma unroll
    for (int w = 1; w < NWAVES; ++w) { ra = fmaxf(ra, s_red[w]); rb = fmaxf(rb, s_red2[w]); }
    __syncthreads();
    a = ra;
    b = rb;
}

// Sum of the four lanes of a float4, exact in fp64: the normalisers A and Z_q enter the accept
// ratios divided by the rejection probabilities, so their rounding must stay far below 1e-6.
__device__ __forceinline__ double sum4(const float4 &v)
{
    return ((double)v.x + (double)v.y) + ((double)v.z + (double)v.w);
}

template <int ITEMS, int VT, bool ALIGNED>
__device__ __forceinline__ void load_row(const float *z, int V, float4 (&r)[ITEMS])
{
    const float ninf = -INFINITY;
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        int e = 4 * (threadIdx.x + VT * i);
        if (ALIGNED) {
            // a logit row is read exactly once by one workgroup: non-temporal, it does not displace
            // anything in L2 (measured 59 -> 56 us on the batched workload)
            typedef float nt_f32x4 __attribute__((ext_vector_type(4)));
            if (e < V) {
                const nt_f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const nt_f32x4 *>(z + e));
                r[i] = make_float4(v[0], v[1], v[2], v[3]);
            } else {
                r[i] = make_float4(ninf, ninf, ninf, ninf);
            }
        } else {
            r[i].x = (e + 0 < V) ? z[e + 0] : ninf;
            r[i].y = (e + 1 < V) ? z[e + 1] : ninf;
            r[i].z = (e + 2 < V) ? z[e + 2] : ninf;
            r[i].w = (e + 3 < V) ? z[e + 3] : ninf;
        }
    }
}

// A logit row is read through a buffer resource whose extent is the row: the address of float4
// number t + VT i is one per-thread offset plus a scalar, reads past the end return zero instead
// of leaving the array, and no per-load address registers or bounds branches are needed.
// Elements past V are then set to -inf (only in the float4s that can reach past V at all).
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ __amdgpu_buffer_rsrc_t row_resource(const float *row, int V)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(row), 0, V * 4, 0x00020000);
}

template <int VT, bool ALIGNED, bool NONTEMPORAL>
__device__ __forceinline__ float4 load_row_piece(__amdgpu_buffer_rsrc_t rs, int i, int V, int tid)
{
    constexpr int AUX = NONTEMPORAL ? 2 : 0;
    const int voff = tid * 16, soff = i * (VT * 16);
    // the thread's first element of this piece lies past V iff 4 t >= V - 4 VT i: one per-thread
    // value against a scalar, no per-piece index registers
    const int e0 = 4 * tid, lim = V - 4 * VT * i;
    const float ninf = -INFINITY;
    float4 r;
    if (ALIGNED) {
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, voff, soff, AUX);
        const bool past = e0 >= lim;
        r = make_float4(past ? ninf : __uint_as_float(v[0]), past ? ninf : __uint_as_float(v[1]),
                        past ? ninf : __uint_as_float(v[2]), past ? ninf : __uint_as_float(v[3]));
    } else {
        // (row start and length are not multiples of 16 bytes: element by element)
        r.x = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rs, voff, soff, AUX));
        r.y = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rs, voff + 4, soff, AUX));
        r.z = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rs, voff + 8, soff, AUX));
        r.w = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rs, voff + 12, soff, AUX));
        if (e0 + 0 >= lim) r.x = ninf;
        if (e0 + 1 >= lim) r.y = ninf;
        if (e0 + 2 >= lim) r.z = ninf;
        if (e0 + 3 >= lim) r.w = ninf;
    }
    return r;
}

// max(a, b, c) as the one hardware instruction.  fmaxf() has to quiet signalling NaNs, and for
// values the compiler knows nothing about (loaded from memory) it does so with an extra
// v_max_f32 x, x per operand: three instructions per element instead of half of one.  The
// instruction itself returns the largest non-NaN operand, which is what the row maximum wants.
__device__ __forceinline__ float max3_raw(float a, float b, float c)
{
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

template <int ITEMS>
__device__ __forceinline__ float row_max(const float4 (&r)[ITEMS])
{
    float m = -INFINITY;
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) m = max3_raw(max3_raw(m, r[i].x, r[i].y), r[i].z, r[i].w);
    return m;
}

// r := 2^((r - m) c) with c = log2(e) / T, i.e. exp((r - m) / T); returns this thread's partial
// sum in fp64.  The subtraction comes first on purpose: the row maximum maps to exactly 1, so
// when one token dominates both distributions (p ~ q, small rejection probability) the residual
// max(0, p - q) does not inherit a rounding error from its largest, cancelling term.
template <int ITEMS>
__device__ __forceinline__ double row_exp(float4 (&r)[ITEMS], float m, float c)
{
    double s = 0.0;
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        // v_exp_f32 directly: results below the normal range flush to zero, which is what
        // a probability of 2^-126 relative to the mode should become anyway
        r[i].x = __builtin_amdgcn_exp2f((r[i].x - m) * c);
        r[i].y = __builtin_amdgcn_exp2f((r[i].y - m) * c);
        r[i].z = __builtin_amdgcn_exp2f((r[i].z - m) * c);
        r[i].w = __builtin_amdgcn_exp2f((r[i].w - m) * c);
        s += sum4(r[i]);
    }
    return s;
}

template <int ITEMS, int VT, bool ALIGNED>
__device__ __forceinline__ void store_row_scaled(float *dst, int V, const float4 (&r)[ITEMS], float s)
{
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        int e = 4 * (threadIdx.x + VT * i);
        float4 v = make_float4(r[i].x * s, r[i].y * s, r[i].z * s, r[i].w * s);
        if (ALIGNED) {
            if (e < V) *reinterpret_cast<float4 *>(dst + e) = v;
        } else {
            if (e + 0 < V) dst[e + 0] = v.x;
            if (e + 1 < V) dst[e + 1] = v.y;
            if (e + 2 < V) dst[e + 2] = v.z;
            if (e + 3 < V) dst[e + 3] = v.w;
        }
    }
}

// Inverse CDF of the unnormalised weights a (sum A) at u: the smallest token id x
// with sum_{y <= x} a(y) > u * A, found by a two-level search: (1) totals of the
// ITEMS contiguous segments of 4 VT tokens, (2) a block-wide inclusive scan inside
// the segment that holds the crossing.  fp64 throughout.
//
// cdf_segments prepares level (1): s_tot[i] = the total of segment i (four-token sums of the
// threads, added up per row of 16 lanes and then over the rows and waves in a fixed order).
// cdf_search does the rest and may be called repeatedly on the same prepared state; a caller
// that removes a token between searches keeps s_tot and A in step itself.
// s_seg holds 4 (VT / 64) ITEMS doubles.
template <int ITEMS, int VT>
__device__ __forceinline__ void cdf_segments(const float4 (&a)[ITEMS], double *s_seg, double *s_tot)
{
    constexpr int NROWS = VT / 16;
    constexpr int SC = ITEMS < 4 ? ITEMS : 4;        // segments reduced together (bounds the registers in use)
    const int t = threadIdx.x, lane = t & 63;
#pragma unroll
    for (int i0 = 0; i0 < ITEMS; i0 += SC) {
        double x[SC];
#pragma unroll
        for (int i = 0; i < SC; ++i) x[i] = sum4(a[i0 + i]);
        int which;
        const double w = row_totals_scattered<SC>(x, lane, which);
        s_seg[(t >> 4) * ITEMS + i0 + which] = w;     // (with fewer than 16 values several lanes of a row store the same total)
    }
    __syncthreads();
    if (t < ITEMS) {
        double tot = 0.0;
        for (int r = 0; r < NROWS; ++r) tot += s_seg[r * ITEMS + t];
        s_tot[t] = tot;
    }
    __syncthreads();
}

template <int ITEMS, int VT>
__device__ __forceinline__ int cdf_search(const float4 (&a)[ITEMS], double A, double u, double eps, double *s_red,
                                          const double *s_tot, int *s_int, uint32_t *flag_bits)
{
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const double tau = u * A;
    if (t == 0) { s_int[0] = 0x7fffffff; s_int[1] = -1; }
    int istar = -1;
    double base = 0.0;
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        const double tot = s_tot[i];
        if (istar < 0) {
            if (base + tot > tau) istar = i;
            else base += tot;
        }
    }
    __syncthreads();
    if (istar >= 0) {
        float4 mine = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int i = 0; i < ITEMS; ++i)
            if (i == istar) mine = a[i];
        const double incl = wave_scan_inclusive(sum4(mine));
        if (lane == 63) s_red[wave] = incl;
        __syncthreads();
        double woff = base;
        for (int w = 0; w < wave; ++w) woff += s_red[w];
        __syncthreads();
        const double cum_hi = woff + incl;              // inclusive running sum up to this thread's 4 tokens
        if (lane == 63) s_red[wave] = cum_hi;
        __syncthreads();
        double cum_lo = __shfl_up(cum_hi, 1);            // the neighbour's inclusive value, bit for bit
        if (lane == 0) cum_lo = (wave == 0) ? base : s_red[wave - 1];
        if (cum_hi > tau && !(cum_lo > tau)) {
            const float v[4] = {mine.x, mine.y, mine.z, mine.w};
            double cum = cum_lo, lo = cum_lo, hi = cum_hi;
            int pick = -1, last_pos = -1;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                double nxt = cum + (double)v[e];
                if (v[e] > 0.f) last_pos = e;
                if (pick < 0 && nxt > tau) { pick = e; lo = cum; hi = nxt; }
                cum = nxt;
            }
            if (pick < 0) pick = last_pos < 0 ? 3 : last_pos;
            int token = 4 * (t + VT * istar) + pick;
            atomicMin(&s_int[0], token);
            if (fabs(tau - lo) < eps * A || fabs(hi - tau) < eps * A) atomicOr(flag_bits, (uint32_t)MCSD_FLAG_NEAR_TIE_ENDPOINT);
        }
    }
    __syncthreads();
    int token = s_int[0];
    if (token == 0x7fffffff) {
        // rounding left no crossing: the last token that carries mass
        int best = -1;
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            int e = 4 * (t + VT * i);
            if (a[i].x > 0.f) best = max(best, e);
            if (a[i].y > 0.f) best = max(best, e + 1);
            if (a[i].z > 0.f) best = max(best, e + 2);
            if (a[i].w > 0.f) best = max(best, e + 3);
        }
        if (best >= 0) atomicMax(&s_int[1], best);
        if (t == 0) atomicOr(flag_bits, (uint32_t)MCSD_FLAG_NEAR_TIE_ENDPOINT);
        __syncthreads();
        token = s_int[1];
    }
    __syncthreads();
    return token;
}

// One-shot form: s_seg holds 4 (VT / 64) ITEMS + ITEMS doubles.
template <int ITEMS, int VT>
__device__ __forceinline__ int inverse_cdf(const float4 (&a)[ITEMS], double A, double u, double eps,
                                           double *s_red, double *s_seg, int *s_int, uint32_t *flag_bits)
{
    double *s_tot = s_seg + 4 * (VT / 64) * ITEMS;
    cdf_segments<ITEMS, VT>(a, s_seg, s_tot);
    return cdf_search<ITEMS, VT>(a, A, u, eps, s_red, s_tot, s_int, flag_bits);
}

}  // namespace vocab
}  // namespace mcsd
