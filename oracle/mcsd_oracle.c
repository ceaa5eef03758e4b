/*
 * CPU oracle for the verification step of Multi-Candidate Speculative Decoding.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference the GPU
 * library is checked against.  It shares no code, header, table or helper with
 * the HIP path, and nothing in the product path may call it (only tests/, the
 * smoke check and the cpu_baseline leg of the bench do).
 *
 * Everything is computed in fp64 from inputs converted exactly out of their
 * storage type (fp32, or bf16 bit patterns).  Loops follow the definitions in
 * the order the paper states them; there is no blocking, fusion or reordering.
 * OpenMP is used only across independent units (one query row, one tree node).
 *
 * What each function follows:
 *   mcsd_oracle_tree_attn      Sec. 3.3 (Tree Attention) and the caption of its
 *                              figure: softmax attention in which a candidate
 *                              sees the whole shared prefix, its ancestors and
 *                              itself.
 *   mcsd_oracle_verify_parent  Algorithm 1 (candidates drawn with replacement)
 *                              and Algorithm 2 (without replacement, q-bar of
 *                              Eq. (1)); the k=1 case is the speculative
 *                              sampling rule of Sec. 2.
 *                              Variant 2 is multi-candidate naive sampling, the
 *                              comparison rule of the ablation (Sec. 4.5, footnote;
 *                              naive sampling of Sec. 2 for k = 1).
 *   mcsd_oracle_verify         Sec. 3, the paragraph describing verification as
 *                              a walk from the root of the candidate tree to a
 *                              leaf, with the endpoint rules of Sec. 2.
 *   mcsd_oracle_draft_parent / mcsd_oracle_draft_sample
 *                              Sec. 3.1, the k candidates sampled from the draft
 *                              distribution at each step: independent draws
 *                              (input of Algorithm 1) or sequential draws without
 *                              replacement from q-bar of Eq. (1) (input of
 *                              Algorithm 2).
 *   mcsd_oracle_tree_build     Sec. 3 / Sec. 4.3: the k-ary candidate tree of a
 *                              k-configuration in generation order (Sec. 3.3).
 *   mcsd_oracle_kv_commit      Sec. 3.3: keys and values of generated tokens are
 *                              cached; the accepted path joins the prefix cache.
 *
 * Pins (tests/test_oracle_*.py): exact enumeration of the output distribution
 * against the theorems of Appendix A and B, the per-round accept / reject
 * masses of Appendix A, hand-derived rational examples, the k=1 textbook rule,
 * the Appendix C inequality, the argmax behaviour stated in Sec. 4.5, and
 * brute-force per-path causal attention; for the draft sampler the measure of
 * the uniforms mapped to each candidate tuple against q and Eq. (1), numpy's
 * cumulative-sum search, and the end-to-end law (sampler + Algorithm 1 / 2
 * returns the target distribution); for the tree builder a queue-based
 * construction and the level-size products; for the KV commit textbook
 * attention over the committed cache against tree attention of the accepted
 * node.  No function here is unpinned.
 *
 * Readings taken where the paper is silent (listed in full in the design notes
 * of this repository): self is attendable; the root is the last context token
 * and is not a query row; accept iff u <= min(1, p/q); q(x)=0 gives ratio 1 if
 * p(x)>0 else 0; a zero residual mass leaves p unchanged; the endpoint is drawn
 * by inverse CDF in token-id order from one supplied uniform; ties in argmax go
 * to the lowest id; Algorithm 2's residual uses q before the rejected token is
 * removed (as in Appendix B's definition of p-bar_n).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_FP32 0
#define ORACLE_BF16 1

#define VARIANT_WITH_REPLACEMENT 0
#define VARIANT_WITHOUT_REPLACEMENT 1
#define VARIANT_NAIVE 2 /* multi-candidate naive sampling (Sec. 4.5, footnote; Sec. 2 for k = 1) */

static double load_elem(const void *base, int dtype, size_t idx)
{
    if (dtype == ORACLE_FP32)
        return (double)((const float *)base)[idx];
    uint32_t bits = (uint32_t)((const uint16_t *)base)[idx] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

int mcsd_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------ attention
 * One output row: query (b, node, head) attends to prefix keys 0..L_b-1 and to
 * the tree keys in A(node) = {node} U A(parent[node]), A(-1) = {} (Sec. 3.3).
 * q        [B][N][H_q][d]
 * k_prefix [B][H_kv][L_stride][d], v_prefix same
 * k_tree   [B][H_kv][N][d],        v_tree   same
 * The KV head of query head h is h / (H_q / H_kv).
 */
static void attn_one_row(int b, int node, int h, int N, int H_q, int H_kv, int d, int dtype,
                         long L_stride, double scale, const void *q, const void *k_prefix,
                         const void *v_prefix, const int32_t *prefix_len, const void *k_tree,
                         const void *v_tree, const int32_t *parent, double *out)
{
    int g = h / (H_q / H_kv);
    long L = prefix_len[b];
    /* ancestor set, self included */
    int *anc = (int *)malloc(sizeof(int) * (size_t)(N > 0 ? N : 1));
    int n_anc = 0;
    for (int a = node; a >= 0; a = parent[a])
        anc[n_anc++] = a;
    long n_keys = L + n_anc;
    double *s = (double *)malloc(sizeof(double) * (size_t)n_keys);
    size_t q_off = (((size_t)b * N + node) * H_q + h) * (size_t)d;
    size_t pre_off = ((size_t)b * H_kv + g) * (size_t)L_stride * d;
    size_t tree_off = ((size_t)b * H_kv + g) * (size_t)N * d;

    for (long j = 0; j < L; ++j) {
        double acc = 0.0;
        for (int c = 0; c < d; ++c)
            acc += load_elem(q, dtype, q_off + c) * load_elem(k_prefix, dtype, pre_off + (size_t)j * d + c);
        s[j] = scale * acc;
    }
    for (int t = 0; t < n_anc; ++t) {
        double acc = 0.0;
        for (int c = 0; c < d; ++c)
            acc += load_elem(q, dtype, q_off + c) * load_elem(k_tree, dtype, tree_off + (size_t)anc[t] * d + c);
        s[L + t] = scale * acc;
    }
    double m = -INFINITY;
    for (long j = 0; j < n_keys; ++j)
        if (s[j] > m) m = s[j];
    double denom = 0.0;
    for (long j = 0; j < n_keys; ++j) {
        s[j] = exp(s[j] - m);
        denom += s[j];
    }
    for (int c = 0; c < d; ++c) {
        double acc = 0.0;
        for (long j = 0; j < L; ++j)
            acc += s[j] * load_elem(v_prefix, dtype, pre_off + (size_t)j * d + c);
        for (int t = 0; t < n_anc; ++t)
            acc += s[L + t] * load_elem(v_tree, dtype, tree_off + (size_t)anc[t] * d + c);
        out[c] = acc / denom;
    }
    free(s);
    free(anc);
}

/* sel == NULL: all rows, out is [B][N][H_q][d].
 * sel != NULL: n_sel triples (b, node, head), out is [n_sel][d]. */
int mcsd_oracle_tree_attn(int B, int N, int H_q, int H_kv, int d, int dtype, long L_stride,
                          double scale, const void *q, const void *k_prefix, const void *v_prefix,
                          const int32_t *prefix_len, const void *k_tree, const void *v_tree,
                          const int32_t *parent, const int32_t *sel, long n_sel, double *out,
                          int n_threads)
{
    if (B < 0 || N < 0 || H_q <= 0 || H_kv <= 0 || H_q % H_kv != 0 || d <= 0)
        return -1;
    for (int i = 0; i < N; ++i)
        if (parent[i] < -1 || parent[i] >= i)
            return -2;
    long total = sel ? n_sel : (long)B * N * H_q;
    if (n_threads < 1) n_threads = 1;
#pragma omp parallel for schedule(dynamic, 1) num_threads(n_threads)
    for (long r = 0; r < total; ++r) {
        int b, node, h;
        if (sel) {
            b = sel[3 * r]; node = sel[3 * r + 1]; h = sel[3 * r + 2];
        } else {
            b = (int)(r / ((long)N * H_q));
            node = (int)((r / H_q) % N);
            h = (int)(r % H_q);
        }
        attn_one_row(b, node, h, N, H_q, H_kv, d, dtype, L_stride, scale, q, k_prefix, v_prefix,
                     prefix_len, k_tree, v_tree, parent, out + (size_t)r * d);
    }
    return 0;
}

/* --------------------------------------------------------------- verification */
static void softmax_T(const float *z, int V, double T, double *p)
{
    double m = -INFINITY;
    for (int x = 0; x < V; ++x) {
        double t = (double)z[x] / T;
        if (t > m) m = t;
    }
    double sum = 0.0;
    for (int x = 0; x < V; ++x) {
        p[x] = exp((double)z[x] / T - m);
        sum += p[x];
    }
    for (int x = 0; x < V; ++x)
        p[x] /= sum;
}

static int argmax_lowest(const float *z, int V)
{
    int best = 0;
    for (int x = 1; x < V; ++x)
        if (z[x] > z[best]) best = x;
    return best;
}

/* Smallest x with sum_{y<=x} p(y) > u; if rounding leaves none, the largest x
 * with p(x) > 0.  *margin receives the distance from u to the nearer edge of
 * the chosen token's CDF interval. */
static int inverse_cdf(const double *p, int V, double u, double *margin)
{
    double cdf = 0.0;
    int last_pos = -1;
    for (int x = 0; x < V; ++x) {
        double lo = cdf;
        cdf += p[x];
        if (p[x] > 0.0) last_pos = x;
        if (cdf > u) {
            double m_lo = fabs(u - lo), m_hi = fabs(cdf - u);
            *margin = m_lo < m_hi ? m_lo : m_hi;
            return x;
        }
    }
    *margin = fabs(u - cdf);
    return last_pos < 0 ? V - 1 : last_pos;
}

/*
 * Algorithm 1 / Algorithm 2 for one parent.
 *   z_p, z_q   logit rows [V]; p = softmax(z_p / T), q = softmax(z_q / T)
 *   tok[k]     candidate ids in sampling order;  u_acc[k] their uniforms
 *   u_end      uniform for the endpoint draw
 *   T == 0     argmax behaviour (Sec. 4.5): accept the first candidate equal to
 *              argmax z_p, otherwise the endpoint is that argmax; z_q, uniforms
 *              unused.  k == 0 is a leaf: endpoint ~ softmax(z_p / T).
 * Outputs: *accepted = index in 0..k-1 of the accepted candidate or -1;
 *   *endpoint = endpoint token when nothing was accepted, else -1;
 *   ratio[k] = min(1, p/q) actually tested, NaN for candidates not reached;
 *   *margin = smallest |uniform - threshold| over the decisions taken;
 *   residual[V] (nullable) = the distribution p held when the loop ended.
 */
int mcsd_oracle_verify_parent(int V, int k, int variant, double T, const float *z_p,
                              const float *z_q, const int32_t *tok, const float *u_acc,
                              double u_end, int32_t *accepted, int32_t *endpoint, double *ratio,
                              double *margin, double *residual)
{
    *accepted = -1;
    *endpoint = -1;
    *margin = INFINITY;
    for (int i = 0; i < k; ++i)
        ratio[i] = NAN;

    if (T == 0.0) {
        int g = argmax_lowest(z_p, V);
        for (int i = 0; i < k; ++i)
            if (tok[i] == g) {
                *accepted = i;
                break;
            }
        if (*accepted < 0) *endpoint = g;
        if (residual) {
            for (int x = 0; x < V; ++x) residual[x] = 0.0;
            residual[g] = 1.0;
        }
        return 0;
    }

    double *p = (double *)malloc(sizeof(double) * (size_t)V);
    double *q = (double *)malloc(sizeof(double) * (size_t)V);
    softmax_T(z_p, V, T, p);

    if (variant == VARIANT_NAIVE) {
        /* multi-candidate naive sampling: a token x is drawn from p first (with the endpoint
         * uniform); a candidate is accepted iff it equals x (the first such), otherwise the
         * candidates are rejected and x is returned.  q and the accept uniforms are not used. */
        double mg;
        int x = inverse_cdf(p, V, u_end, &mg);
        *margin = mg;
        for (int i = 0; i < k; ++i) {
            if (tok[i] < 0 || tok[i] >= V) { free(p); free(q); return -3; }
            if (*accepted < 0 && tok[i] == x) *accepted = i;
        }
        if (*accepted < 0) *endpoint = x;
        if (residual) memcpy(residual, p, sizeof(double) * (size_t)V);
        free(p);
        free(q);
        return 0;
    }
    if (k > 0) softmax_T(z_q, V, T, q);

    for (int i = 0; i < k; ++i) {
        int x = tok[i];
        if (x < 0 || x >= V) {
            free(p); free(q);
            return -3;
        }
        double r = (double)u_acc[i];
        double rat;
        if (q[x] > 0.0) {
            rat = p[x] / q[x];
            if (rat > 1.0) rat = 1.0;
        } else {
            rat = p[x] > 0.0 ? 1.0 : 0.0;
        }
        ratio[i] = rat;
        double mg = fabs(r - rat);
        if (mg < *margin) *margin = mg;
        /* a token of probability zero is never accepted (Sec. 3.2: a rejected token has residual
         * probability 0), also not by a uniform of exactly 0 from outside the open interval */
        if (rat > 0.0 && r <= rat) {
            *accepted = i;
            break;
        }
        /* rejected: p := max(0, p - q) / sum max(0, p - q), with the q of this
         * round (Appendix B defines p-bar_n from q-bar_{n-1}) */
        double S = 0.0;
        for (int y = 0; y < V; ++y) {
            double w = p[y] - q[y];
            S += w > 0.0 ? w : 0.0;
        }
        if (S > 0.0) {
            for (int y = 0; y < V; ++y) {
                double w = p[y] - q[y];
                p[y] = (w > 0.0 ? w : 0.0) / S;
            }
        } /* else: impossible after a rejection in exact arithmetic; p is left unchanged */
        if (variant == VARIANT_WITHOUT_REPLACEMENT) {
            q[x] = 0.0;
            double sq = 0.0;
            for (int y = 0; y < V; ++y) sq += q[y];
            if (sq > 0.0)
                for (int y = 0; y < V; ++y) q[y] /= sq;
        }
    }

    if (*accepted < 0) {
        double mg;
        *endpoint = inverse_cdf(p, V, u_end, &mg);
        if (mg < *margin) *margin = mg;
    }
    if (residual) memcpy(residual, p, sizeof(double) * (size_t)V);
    free(p);
    free(q);
    return 0;
}

/*
 * Whole step: every row owner (root row 0, node i -> row 1+i) is evaluated, then
 * the walk of Sec. 3 picks the path.
 *   target_logits [B][1+N][V], draft_logits [B][P][V], q_row [1+N] (-1: leaf)
 *   parent [N], cand_tok [B][N], u_accept [B][N], u_endpoint [B][1+N], temperature [B]
 * Per-row outputs: acc_child [B][1+N] (node id or -1), endpoint [B][1+N] (-1 when a
 *   child was accepted), ratio [B][N], margin [B][1+N], residual [B][1+N][V] or NULL.
 * Walk outputs: n_accepted [B], accepted_path [B][gamma_max] (-1 padded),
 *   out_tokens [B][gamma_max+1] (accepted tokens then the endpoint, -1 padded).
 */
int mcsd_oracle_verify(int B, int N, int V, int P, int variant, const float *target_logits,
                       const float *draft_logits, const int32_t *q_row, const int32_t *parent,
                       const int32_t *cand_tok, const float *u_accept, const float *u_endpoint,
                       const float *temperature, int32_t *acc_child, int32_t *endpoint,
                       double *ratio, double *margin, double *residual, int32_t *n_accepted,
                       int32_t *accepted_path, int32_t *out_tokens, int gamma_max, int n_threads)
{
    for (int i = 0; i < N; ++i)
        if (parent[i] < -1 || parent[i] >= i) return -2;
    for (int r = 0; r <= N; ++r)
        if (q_row[r] >= P) return -1;
    if (n_threads < 1) n_threads = 1;
    int status = 0;
    long rows = (long)B * (1 + N);
    for (long i = 0; i < (long)B * N; ++i) ratio[i] = NAN;

#pragma omp parallel for schedule(dynamic, 1) num_threads(n_threads)
    for (long r = 0; r < rows; ++r) {
        int b = (int)(r / (1 + N));
        int row = (int)(r % (1 + N));
        int v = row - 1; /* node id, -1 for the root */
        int kids[1024];
        int k = 0;
        for (int i = 0; i < N && k < 1024; ++i)
            if (parent[i] == v) kids[k++] = i;
        int32_t toks[1024];
        float us[1024];
        double rat[1024];
        for (int i = 0; i < k; ++i) {
            toks[i] = cand_tok[(size_t)b * N + kids[i]];
            us[i] = u_accept[(size_t)b * N + kids[i]];
        }
        const float *zp = target_logits + ((size_t)b * (1 + N) + row) * V;
        const float *zq = (k > 0 && q_row[row] >= 0)
                              ? draft_logits + ((size_t)b * P + q_row[row]) * V
                              : zp;
        int32_t acc, endp;
        double mg;
        int rc = mcsd_oracle_verify_parent(V, k, variant, (double)temperature[b], zp, zq, toks, us,
                                           (double)u_endpoint[(size_t)b * (1 + N) + row], &acc,
                                           &endp, rat, &mg,
                                           residual ? residual + (size_t)r * V : NULL);
        if (rc != 0) {
#pragma omp critical
            status = rc;
        }
        acc_child[r] = acc >= 0 ? kids[acc] : -1;
        endpoint[r] = endp;
        margin[r] = mg;
        for (int i = 0; i < k; ++i)
            ratio[(size_t)b * N + kids[i]] = rat[i];
    }
    if (status != 0) return status;

    for (int b = 0; b < B; ++b) {
        for (int i = 0; i < gamma_max; ++i) accepted_path[(size_t)b * gamma_max + i] = -1;
        for (int i = 0; i <= gamma_max; ++i) out_tokens[(size_t)b * (gamma_max + 1) + i] = -1;
        int row = 0, n = 0;
        for (;;) {
            size_t r = (size_t)b * (1 + N) + row;
            int c = acc_child[r];
            if (c >= 0 && n >= gamma_max) return -4; /* tree deeper than gamma_max */
            if (c < 0) {
                /* all candidates rejected, or a leaf: the endpoint closes the block */
                out_tokens[(size_t)b * (gamma_max + 1) + n] = endpoint[r];
                break;
            }
            accepted_path[(size_t)b * gamma_max + n] = c;
            out_tokens[(size_t)b * (gamma_max + 1) + n] = cand_tok[(size_t)b * N + c];
            ++n;
            row = 1 + c;
        }
        n_accepted[b] = n;
    }
    return 0;
}

/* ------------------------------------------------------- draft-side candidates
 *
 * The k candidates of one parent, drawn from the draft distribution
 * q = softmax(z_q / T) (Sec. 3.1: the batch of candidates sampled at each step).
 *   variant 0 (Algorithm 1's input): k independent draws from q;
 *   variant 1 (Algorithm 2's input): sequentially without replacement, draw i
 *     from q-bar of Eq. (1): q with the earlier draws zeroed, renormalised;
 *   T == 0: the k largest logits in descending order, lowest id on ties (k
 *     distinct candidates of a draft model that samples by arg max).
 * Draw i uses the supplied uniform u[i] by inverse CDF in token-id order (the
 * same convention as the endpoint draw above).  margin[i] = distance from u[i]
 * to the nearer edge of the chosen token's CDF interval (infinity for T == 0).
 */
int mcsd_oracle_draft_parent(int V, int k, int variant, double T, const float *z_q,
                             const float *u, int32_t *tok, double *margin)
{
    if (V <= 0 || k < 0 || k > V) return -1;
    if (T == 0.0) {
        char *taken = (char *)calloc((size_t)V, 1);
        if (!taken) return -3;
        for (int i = 0; i < k; ++i) {
            int best = -1;
            for (int x = 0; x < V; ++x)
                if (!taken[x] && (best < 0 || z_q[x] > z_q[best])) best = x;
            taken[best] = 1;
            tok[i] = best;
            margin[i] = INFINITY;
        }
        free(taken);
        return 0;
    }
    double *q = (double *)malloc(sizeof(double) * (size_t)V);
    if (!q) return -3;
    softmax_T(z_q, V, T, q);
    for (int i = 0; i < k; ++i) {
        tok[i] = inverse_cdf(q, V, (double)u[i], &margin[i]);
        if (variant == VARIANT_WITHOUT_REPLACEMENT) {
            q[tok[i]] = 0.0;
            double s = 0.0;
            for (int x = 0; x < V; ++x) s += q[x];
            if (s > 0.0)
                for (int x = 0; x < V; ++x) q[x] /= s;
        }
    }
    free(q);
    return 0;
}

/*
 * Candidates of a whole tree: for every row that has children (root row 0, node i
 * -> row 1+i) the children, in ascending node id, receive the draws of
 * mcsd_oracle_draft_parent from draft row q_row[row].
 *   draft_logits [B][P][V], q_row [1+N], parent [N], u_draw [B][N], temperature [B]
 *   -> cand_tok [B][N], margin [B][N]
 */
int mcsd_oracle_draft_sample(int B, int N, int V, int P, int variant, const float *draft_logits,
                             const int32_t *q_row, const int32_t *parent, const float *u_draw,
                             const float *temperature, int32_t *cand_tok, double *margin,
                             int n_threads)
{
    for (int i = 0; i < N; ++i)
        if (parent[i] < -1 || parent[i] >= i) return -2;
    if (n_threads < 1) n_threads = 1;
    int status = 0;
    long rows = (long)B * (1 + N);
#pragma omp parallel for schedule(dynamic, 1) num_threads(n_threads)
    for (long r = 0; r < rows; ++r) {
        int b = (int)(r / (1 + N));
        int row = (int)(r % (1 + N));
        int kids[1024];
        int k = 0;
        for (int i = 0; i < N && k < 1024; ++i)
            if (parent[i] == row - 1) kids[k++] = i;
        if (k == 0) continue;
        int rc = 0;
        if (q_row[row] < 0 || q_row[row] >= P) {
            rc = -1;
        } else {
            float us[1024];
            int32_t toks[1024];
            double mg[1024];
            for (int i = 0; i < k; ++i) us[i] = u_draw[(size_t)b * N + kids[i]];
            rc = mcsd_oracle_draft_parent(V, k, variant, (double)temperature[b],
                                          draft_logits + ((size_t)b * P + q_row[row]) * V, us, toks, mg);
            if (rc == 0)
                for (int i = 0; i < k; ++i) {
                    cand_tok[(size_t)b * N + kids[i]] = toks[i];
                    margin[(size_t)b * N + kids[i]] = mg[i];
                }
        }
        if (rc != 0) {
#pragma omp critical
            status = rc;
        }
    }
    return status;
}

/* ------------------------------------------------ candidate tree and KV commit
 *
 * mcsd_oracle_tree_build: the k-ary candidate tree of a k-configuration
 * (k_1, ..., k_gamma) (Sec. 3, verification as a walk over the k branches of a
 * tree; Sec. 4.3 for the k-configuration), laid out in generation order as
 * Sec. 3.3 packs the candidates into one sequence: level by level, every node
 * of level i-1 (the root for i = 1) receives k_i children, the children of one
 * parent are consecutive.  Node ids exclude the root.
 *   parent[N] (-1: child of the root), depth[N] (1-based), q_row[1+N] (index of
 *   the draft row of every tree row that has children, in row order; -1 for the
 *   leaves).  Returns N, or -1 if a k_i is < 1 or N would exceed max_nodes.
 */
int mcsd_oracle_tree_build(const int32_t *kconfig, int gamma, int max_nodes, int32_t *parent,
                           int32_t *depth, int32_t *q_row)
{
    int n = 0;
    int level_begin = -1, level_count = 1; /* the root alone forms level 0 */
    for (int lvl = 1; lvl <= gamma; ++lvl) {
        int k = kconfig[lvl - 1];
        if (k < 1) return -1;
        int first = n;
        for (int j = 0; j < level_count; ++j) {
            int par = (lvl == 1) ? -1 : level_begin + j;
            for (int c = 0; c < k; ++c) {
                if (n >= max_nodes) return -1;
                parent[n] = par;
                depth[n] = lvl;
                ++n;
            }
        }
        level_begin = first;
        level_count = n - first;
    }
    int next = 0;
    for (int row = 0; row <= n; ++row) {
        int has_child = 0;
        for (int i = 0; i < n; ++i)
            if (parent[i] == row - 1) has_child = 1;
        q_row[row] = has_child ? next++ : -1;
    }
    return n;
}

/*
 * mcsd_oracle_kv_commit: the keys and values of generated tokens stay unchanged
 * and are cached for reuse (Sec. 3.3); after verification the accepted candidates
 * are generated tokens, so their K/V rows move from the tree block to the tail of
 * the prefix cache, in path order, and the prefix grows by the number accepted.
 * The endpoint token (position n_accepted of out_tokens) is the next step's root.
 *   k/v_prefix [n_layers][B][H_kv][L_stride][d] (in/out), k/v_tree [n_layers][B][H_kv][N][d],
 *   elem_bytes per element; n_accepted [B], accepted_path [B][gamma_max],
 *   out_tokens [B][gamma_max+1]; prefix_len [B] (in/out); next_root [B]; full [B]
 *   (1 where prefix_len + n_accepted would exceed L_stride: nothing is copied and
 *   prefix_len keeps its value).
 * root_row = 1: the root of the tree (the token the previous step ended with) went through the
 *   same forward pass as the candidates, so the tree block has 1 + N rows, row 0 the root's and
 *   row 1 + i candidate i's; generated tokens are then the root and the accepted candidates:
 *   the root's row is appended first, the path after it, and the prefix grows by 1 + n_accepted.
 */
int mcsd_oracle_kv_commit(int n_layers, int B, int N, int H_kv, int d, int elem_bytes, long L_stride,
                          int gamma_max, int root_row, unsigned char *k_prefix, unsigned char *v_prefix,
                          const unsigned char *k_tree, const unsigned char *v_tree,
                          const int32_t *n_accepted, const int32_t *accepted_path,
                          const int32_t *out_tokens, int32_t *prefix_len, int32_t *next_root,
                          int32_t *full)
{
    size_t row = (size_t)d * (size_t)elem_bytes;
    for (int b = 0; b < B; ++b) {
        int n = n_accepted[b];
        if (n < 0 || n > gamma_max) return -1;
        next_root[b] = out_tokens[(size_t)b * (gamma_max + 1) + n];
        long L = prefix_len[b];
        int extra = root_row ? 1 : 0;
        int tree_rows = N + extra;
        full[b] = (L + extra + n > L_stride) ? 1 : 0;
        if (full[b]) continue;
        for (int layer = 0; layer < n_layers; ++layer)
            for (int g = 0; g < H_kv; ++g) {
                if (root_row) {
                    size_t src = ((((size_t)layer * B + b) * H_kv + g) * (size_t)tree_rows + 0) * row;
                    size_t dst = ((((size_t)layer * B + b) * H_kv + g) * (size_t)L_stride + (size_t)L) * row;
                    memcpy(k_prefix + dst, k_tree + src, row);
                    memcpy(v_prefix + dst, v_tree + src, row);
                }
                for (int j = 0; j < n; ++j) {
                    int node = accepted_path[(size_t)b * gamma_max + j];
                    if (node < 0 || node >= N) return -2;
                    size_t src = ((((size_t)layer * B + b) * H_kv + g) * (size_t)tree_rows + (size_t)(extra + node)) * row;
                    size_t dst = ((((size_t)layer * B + b) * H_kv + g) * (size_t)L_stride + (size_t)(L + extra + j)) * row;
                    memcpy(k_prefix + dst, k_tree + src, row);
                    memcpy(v_prefix + dst, v_tree + src, row);
                }
            }
        prefix_len[b] = (int32_t)(L + extra + n);
    }
    return 0;
}
