/*
 * ape_oracle.c -- plain fp64 CPU oracle for the APE attention hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may call this file;
 * it exists so that the GPU kernels can be compared with a slow, obviously
 * correct implementation of what the paper defines.  It shares no code,
 * header, table or helper with the HIP library.
 *
 * What is computed (APE paper, arXiv 2502.05431):
 *   - ape_oracle_attention       Section 4.4, the refined attention equation
 *                                ("Eq.5"): prefix + temperature-scaled context
 *                                raised to the power S + the query's own
 *                                causal KV.  Weights form, one weighted sum.
 *   - ape_oracle_attention_hier  Appendix C ("Formal Derivation"): the same
 *                                result built from per-block softmax outputs
 *                                and LogSumExp values, merged by a softmax
 *                                over the LogSumExps.  mode 0 pools all
 *                                contexts into one block before S is applied
 *                                (C.3 / C.4, equal to Eq.5); mode 1 applies S
 *                                to each context's LogSumExp separately (C.2
 *                                as literally written).
 *   - ape_oracle_attention_tree  Appendix C.2 applied recursively to a tree of
 *                                contexts (Appendix C.5): every node merges
 *                                its children by a softmax over their
 *                                LogSumExps and multiplies its own by S_n.
 *   - ape_oracle_rope            rotary position embedding with the positions
 *                                re-used across contexts (Section 1), the step
 *                                that produces the rotated Q/K the attention
 *                                routines read.
 *   - ape_oracle_encode          Section 2.2 "Pre-caching Contexts" with the
 *                                shared prefix of Section 4.1: every context
 *                                row attends causally to the prefix and to
 *                                its own context only (Section 2.3 softmax
 *                                attention, no T, no S).
 *
 * Conventions (layouts are the same as the library's so that the same seeded
 * arrays feed both): every K/V/Q array is row-major [tokens, heads, head_dim],
 * inputs are float (they carry fp32 or bf16-rounded values exactly) and every
 * bit of arithmetic is done in double.  Query head h reads KV head
 * h / (n_q_heads / n_kv_heads).  Natural logarithm everywhere.  Query row r of
 * q_len rows sees self tokens 0 .. self_len - q_len + r (causal; the last
 * q_len self tokens are the query rows themselves).
 *
 * Parallelism: OpenMP over independent (row, head) pairs only.  No blocking,
 * tiling, fusion or reordering of the arithmetic.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* q . k over head_dim, accumulated in double */
static double dot_fd(const float *a, const float *b, int d)
{
    double s = 0.0;
    for (int c = 0; c < d; ++c) s += (double)a[c] * (double)b[c];
    return s;
}

/* log(sum_j exp(x_j)) for n >= 1 values; -inf for n == 0 */
static double logsumexp(const double *x, long n)
{
    if (n <= 0) return -INFINITY;
    double m = x[0];
    for (long j = 1; j < n; ++j) if (x[j] > m) m = x[j];
    if (!(m > -INFINITY)) return -INFINITY;
    double z = 0.0;
    for (long j = 0; j < n; ++j) z += exp(x[j] - m);
    return m + log(z);
}

int ape_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Section 4.4, refined attention (Eq.5), weights form.
 *
 * For one query vector q:
 *   a_P[j]   = exp(q.k_P[j] / sqrt(d))                      prefix
 *   a'_C[t]  = exp(q.k_C[t] / (T sqrt(d)))                  every context token
 *   a[j]     = exp(q.k_self[j] / sqrt(d)),  j causal        query / generated
 *   Z_C      = sum_t a'_C[t]
 *   D        = sum a_P + Z_C^S + sum a
 *   weight of a prefix/self token = a / D
 *   weight of a context token     = a'_C[t] * Z_C^(S-1) / D
 *   O = sum of weight * value over all three parts.
 *
 * The exponentials are evaluated with shifts so that nothing overflows:
 *   a'_C[t] Z_C^(S-1) = exp(s_C[t] - L_C) * exp(S L_C),  L_C = log Z_C,
 * and every term of D carries the common factor exp(-g),
 *   g = max(max s_P, max s_self, S L_C).
 *
 * pair_rows / pair_heads select the (row, head) pairs to compute (both NULL:
 * all q_len * n_q_heads pairs in row-major (row, head) order).
 * out[p*d + c]; lse[p] = log D; ctx_mass[p] = Z_C^S / D (either may be NULL).
 * Returns 0, or -1 on bad arguments.
 */
int ape_oracle_attention(int n_q_heads, int n_kv_heads, int d,
                         const float *k_prefix, const float *v_prefix, int prefix_len,
                         const float *k_ctx, const float *v_ctx,
                         const int *cu_chunk_lens, int n_chunks,
                         const float *k_self, const float *v_self, int self_len,
                         const float *q, int q_len, double T, double S,
                         const int *pair_rows, const int *pair_heads, long n_pairs,
                         double *out, double *lse, double *ctx_mass)
{
    if (n_q_heads <= 0 || n_kv_heads <= 0 || d <= 0 || n_q_heads % n_kv_heads) return -1;
    if (q_len <= 0 || self_len < q_len || prefix_len < 0 || n_chunks < 0) return -1;
    if (!(T > 0.0) || !(S > 0.0)) return -1;
    const int G = n_q_heads / n_kv_heads;
    const long M = n_chunks > 0 ? cu_chunk_lens[n_chunks] : 0;   /* all context tokens */
    const long kv_stride = (long)n_kv_heads * d;
    const double inv_sqrt_d = 1.0 / sqrt((double)d);
    const int all = (pair_rows == NULL);
    if (all) n_pairs = (long)q_len * n_q_heads;
    int bad = 0;

#pragma omp parallel for schedule(dynamic, 1)
    for (long p = 0; p < n_pairs; ++p) {
        const int r = all ? (int)(p / n_q_heads) : pair_rows[p];
        const int h = all ? (int)(p % n_q_heads) : pair_heads[p];
        if (r < 0 || r >= q_len || h < 0 || h >= n_q_heads) { bad = 1; continue; }
        const int hk = h / G;
        const float *qv = q + ((long)r * n_q_heads + h) * d;
        const long n_self = (long)self_len - q_len + r + 1;      /* causal */

        double *sP = (double *)malloc(sizeof(double) * (size_t)(prefix_len + 1));
        double *sC = (double *)malloc(sizeof(double) * (size_t)(M + 1));
        double *sS = (double *)malloc(sizeof(double) * (size_t)(n_self + 1));

        for (long j = 0; j < prefix_len; ++j)
            sP[j] = dot_fd(qv, k_prefix + j * kv_stride + (long)hk * d, d) * inv_sqrt_d;
        for (long t = 0; t < M; ++t)
            sC[t] = dot_fd(qv, k_ctx + t * kv_stride + (long)hk * d, d) * inv_sqrt_d / T;
        for (long j = 0; j < n_self; ++j)
            sS[j] = dot_fd(qv, k_self + j * kv_stride + (long)hk * d, d) * inv_sqrt_d;

        const double L_C = logsumexp(sC, M);                      /* log Z_C, -inf if no context */
        const double ctx_log = (M > 0) ? S * L_C : -INFINITY;     /* log Z_C^S */
        double g = ctx_log;
        for (long j = 0; j < prefix_len; ++j) if (sP[j] > g) g = sP[j];
        for (long j = 0; j < n_self; ++j) if (sS[j] > g) g = sS[j];

        double D = 0.0;                                           /* D * exp(-g) */
        for (long j = 0; j < prefix_len; ++j) D += exp(sP[j] - g);
        if (M > 0) D += exp(ctx_log - g);
        for (long j = 0; j < n_self; ++j) D += exp(sS[j] - g);

        double *o = out + p * d;
        for (int c = 0; c < d; ++c) o[c] = 0.0;
        for (long j = 0; j < prefix_len; ++j) {
            const double w = exp(sP[j] - g) / D;
            const float *vv = v_prefix + j * kv_stride + (long)hk * d;
            for (int c = 0; c < d; ++c) o[c] += w * (double)vv[c];
        }
        for (long t = 0; t < M; ++t) {
            const double w = exp(sC[t] - L_C) * exp(ctx_log - g) / D;
            const float *vv = v_ctx + t * kv_stride + (long)hk * d;
            for (int c = 0; c < d; ++c) o[c] += w * (double)vv[c];
        }
        for (long j = 0; j < n_self; ++j) {
            const double w = exp(sS[j] - g) / D;
            const float *vv = v_self + j * kv_stride + (long)hk * d;
            for (int c = 0; c < d; ++c) o[c] += w * (double)vv[c];
        }
        if (lse) lse[p] = g + log(D);
        if (ctx_mass) ctx_mass[p] = (M > 0) ? exp(ctx_log - g) / D : 0.0;
        free(sP); free(sC); free(sS);
    }
    return bad ? -1 : 0;
}

/* softmax(x) . V for one block of n tokens; returns LogSumExp(x), writes vh[d].
 * (Appendix C.1: the pair (V^h, A^h) of one block.)  n == 0 gives -inf and vh = 0. */
static double block_softmax_value(const double *x, long n, const float *v, long v_stride,
                                  int d, double *vh)
{
    for (int c = 0; c < d; ++c) vh[c] = 0.0;
    const double L = logsumexp(x, n);
    if (n <= 0) return L;
    for (long j = 0; j < n; ++j) {
        const double w = exp(x[j] - L);
        const float *vv = v + j * v_stride;
        for (int c = 0; c < d; ++c) vh[c] += w * (double)vv[c];
    }
    return L;
}

/*
 * Appendix C, hierarchical form.
 *
 * Every block b (prefix+self together, and the context block(s)) yields
 *   V^h_b = Softmax(scores_b) V_b,   A^h_b = LogSumExp(scores_b),
 * context scores carry 1/(T sqrt(d)) and context LogSumExps are multiplied by
 * S; the output is Softmax(A^h_...) applied to the V^h_... (C.1, C.2).
 *   per_context == 0: all contexts form ONE block (C.3 / the C.4 listing:
 *                     one LogSumExp for the whole context part) -> equals Eq.5.
 *   per_context == 1: one block per context, S applied to each (C.2 literal).
 * Prefix and self tokens form one non-context block (C.3 merges them; exact,
 * because blocks with unscaled LogSumExp merge exactly, C.1).
 * Same pair selection and outputs as ape_oracle_attention.
 */
int ape_oracle_attention_hier(int n_q_heads, int n_kv_heads, int d,
                              const float *k_prefix, const float *v_prefix, int prefix_len,
                              const float *k_ctx, const float *v_ctx,
                              const int *cu_chunk_lens, int n_chunks,
                              const float *k_self, const float *v_self, int self_len,
                              const float *q, int q_len, double T, double S, int per_context,
                              const int *pair_rows, const int *pair_heads, long n_pairs,
                              double *out, double *lse)
{
    if (n_q_heads <= 0 || n_kv_heads <= 0 || d <= 0 || n_q_heads % n_kv_heads) return -1;
    if (q_len <= 0 || self_len < q_len || prefix_len < 0 || n_chunks < 0) return -1;
    if (!(T > 0.0) || !(S > 0.0)) return -1;
    const int G = n_q_heads / n_kv_heads;
    const long M = n_chunks > 0 ? cu_chunk_lens[n_chunks] : 0;
    const long kv_stride = (long)n_kv_heads * d;
    const double inv_sqrt_d = 1.0 / sqrt((double)d);
    const int all = (pair_rows == NULL);
    if (all) n_pairs = (long)q_len * n_q_heads;
    const int n_ctx_blocks = (M == 0) ? 0 : (per_context ? n_chunks : 1);
    int bad = 0;

#pragma omp parallel for schedule(dynamic, 1)
    for (long p = 0; p < n_pairs; ++p) {
        const int r = all ? (int)(p / n_q_heads) : pair_rows[p];
        const int h = all ? (int)(p % n_q_heads) : pair_heads[p];
        if (r < 0 || r >= q_len || h < 0 || h >= n_q_heads) { bad = 1; continue; }
        const int hk = h / G;
        const float *qv = q + ((long)r * n_q_heads + h) * d;
        const long n_self = (long)self_len - q_len + r + 1;
        const int nb = n_ctx_blocks + 1;

        double *A = (double *)malloc(sizeof(double) * (size_t)nb);          /* A^h per block */
        double *Vh = (double *)malloc(sizeof(double) * (size_t)nb * d);     /* V^h per block */
        double *x = (double *)malloc(sizeof(double) * (size_t)(M + prefix_len + n_self + 1));

        /* context block(s): temperature in the scores, S on the LogSumExp */
        for (int b = 0; b < n_ctx_blocks; ++b) {
            const long t0 = per_context ? cu_chunk_lens[b] : 0;
            const long t1 = per_context ? cu_chunk_lens[b + 1] : M;
            for (long t = t0; t < t1; ++t)
                x[t - t0] = dot_fd(qv, k_ctx + t * kv_stride + (long)hk * d, d) * inv_sqrt_d / T;
            const double L = block_softmax_value(x, t1 - t0, v_ctx + t0 * kv_stride + (long)hk * d,
                                                 kv_stride, d, Vh + (long)b * d);
            A[b] = S * L;          /* empty context (L = -inf) keeps weight 0 */
        }
        /* non-context block: prefix tokens then the causal self tokens */
        {
            double *vh = Vh + (long)n_ctx_blocks * d;
            double *vp = (double *)malloc(sizeof(double) * (size_t)d);
            double *vs = (double *)malloc(sizeof(double) * (size_t)d);
            for (long j = 0; j < prefix_len; ++j)
                x[j] = dot_fd(qv, k_prefix + j * kv_stride + (long)hk * d, d) * inv_sqrt_d;
            const double LP = block_softmax_value(x, prefix_len, v_prefix + (long)hk * d, kv_stride, d, vp);
            for (long j = 0; j < n_self; ++j)
                x[j] = dot_fd(qv, k_self + j * kv_stride + (long)hk * d, d) * inv_sqrt_d;
            const double LS = block_softmax_value(x, n_self, v_self + (long)hk * d, kv_stride, d, vs);
            /* exact two-block merge (C.1) */
            const double two[2] = { LP, LS };
            const double L = logsumexp(two, 2);
            const double wp = (prefix_len > 0) ? exp(LP - L) : 0.0, ws = exp(LS - L);
            for (int c = 0; c < d; ++c) vh[c] = wp * vp[c] + ws * vs[c];
            A[n_ctx_blocks] = L;
            free(vp); free(vs);
        }
        /* O = Softmax(A^h_...) x [V^h_...] */
        const double Ltot = logsumexp(A, nb);
        double *o = out + p * d;
        for (int c = 0; c < d; ++c) o[c] = 0.0;
        for (int b = 0; b < nb; ++b) {
            if (!(A[b] > -INFINITY)) continue;
            const double w = exp(A[b] - Ltot);
            for (int c = 0; c < d; ++c) o[c] += w * Vh[(long)b * d + c];
        }
        if (lse) lse[p] = Ltot;
        free(A); free(Vh); free(x);
    }
    return bad ? -1 : 0;
}

/*
 * Appendix C.2 applied recursively along a tree of contexts (the tree-shaped
 * cache of Appendix C.5).
 *
 * A node n has a scaling factor S_n and an ordered list of children, which
 * are either all cached contexts (node_leaf[n] != 0: contexts
 * node_first[n] .. node_first[n] + node_count[n] - 1 of the chunk table) or
 * all nodes (node_leaf[n] == 0: nodes node_first[n] .. + node_count[n] - 1,
 * each with an index larger than n).  Node 0 is the root.
 *
 *   context i:  V_i = Softmax(q.K_i / (T sqrt d)) V_i,  A_i = LogSumExp(same scores)
 *   node n:     V_n = Softmax(A_children) [V_children],
 *               A_n = S_n * LogSumExp(A_children)
 *   result:     O = Softmax(A_other, A_root) [V_other, V_root], where "other" is
 *               the unscaled block of prefix + causal self tokens (C.1-C.2).
 *
 * Special cases: a root with scale S over all contexts is the pooled form
 * (C.3, equal to Eq.5); a root with scale 1 over N one-context nodes of scale
 * S is C.2 as literally written.
 */
typedef struct {
    const float *qv;            /* the query vector, d floats */
    const float *k_ctx, *v_ctx; /* packed contexts, already offset to the KV head */
    const int *cu;
    int n_chunks, n_nodes, d;
    long kv_stride;
    double score_scale;         /* 1 / (T sqrt d) */
    const double *node_scale;
    const int *node_first, *node_count, *node_leaf;
    int bad;
} tree_query;

/* writes V_n into vh[d], returns A_n */
static double tree_node_value(tree_query *tq, int n, double *vh)
{
    const int d = tq->d, cnt = tq->node_count[n], first = tq->node_first[n];
    for (int c = 0; c < d; ++c) vh[c] = 0.0;
    if (cnt <= 0) { tq->bad = 1; return -INFINITY; }
    double *A = (double *)malloc(sizeof(double) * (size_t)cnt);
    double *V = (double *)malloc(sizeof(double) * (size_t)cnt * d);
    for (int i = 0; i < cnt; ++i) {
        const int ch = first + i;
        if (tq->node_leaf[n]) {
            if (ch < 0 || ch >= tq->n_chunks) { tq->bad = 1; A[i] = -INFINITY; continue; }
            const long t0 = tq->cu[ch], len = tq->cu[ch + 1] - t0;
            double *x = (double *)malloc(sizeof(double) * (size_t)(len + 1));
            for (long t = 0; t < len; ++t)
                x[t] = dot_fd(tq->qv, tq->k_ctx + (t0 + t) * tq->kv_stride, d) * tq->score_scale;
            A[i] = block_softmax_value(x, len, tq->v_ctx + t0 * tq->kv_stride, tq->kv_stride, d, V + (long)i * d);
            free(x);
        } else {
            if (ch <= n || ch >= tq->n_nodes) { tq->bad = 1; A[i] = -INFINITY; continue; }
            A[i] = tree_node_value(tq, ch, V + (long)i * d);
        }
    }
    const double L = logsumexp(A, cnt);
    if (L > -INFINITY)
        for (int i = 0; i < cnt; ++i) {
            if (!(A[i] > -INFINITY)) continue;
            const double w = exp(A[i] - L);
            for (int c = 0; c < d; ++c) vh[c] += w * V[(long)i * d + c];
        }
    free(A); free(V);
    return tq->node_scale[n] * L;      /* all children empty: stays -inf (S_n > 0) */
}

int ape_oracle_attention_tree(int n_q_heads, int n_kv_heads, int d,
                              const float *k_prefix, const float *v_prefix, int prefix_len,
                              const float *k_ctx, const float *v_ctx,
                              const int *cu_chunk_lens, int n_chunks,
                              const float *k_self, const float *v_self, int self_len,
                              const float *q, int q_len, double T,
                              const double *node_scale, const int *node_first, const int *node_count,
                              const int *node_leaf, int n_nodes,
                              const int *pair_rows, const int *pair_heads, long n_pairs,
                              double *out, double *lse)
{
    if (n_q_heads <= 0 || n_kv_heads <= 0 || d <= 0 || n_q_heads % n_kv_heads) return -1;
    if (q_len <= 0 || self_len < q_len || prefix_len < 0 || n_chunks < 1 || n_nodes < 1) return -1;
    if (!(T > 0.0)) return -1;
    for (int n = 0; n < n_nodes; ++n) if (!(node_scale[n] > 0.0)) return -1;
    const int G = n_q_heads / n_kv_heads;
    const long kv_stride = (long)n_kv_heads * d;
    const double inv_sqrt_d = 1.0 / sqrt((double)d);
    const int all = (pair_rows == NULL);
    if (all) n_pairs = (long)q_len * n_q_heads;
    int bad = 0;

#pragma omp parallel for schedule(dynamic, 1)
    for (long p = 0; p < n_pairs; ++p) {
        const int r = all ? (int)(p / n_q_heads) : pair_rows[p];
        const int h = all ? (int)(p % n_q_heads) : pair_heads[p];
        if (r < 0 || r >= q_len || h < 0 || h >= n_q_heads) { bad = 1; continue; }
        const int hk = h / G;
        const float *qv = q + ((long)r * n_q_heads + h) * d;
        const long n_self = (long)self_len - q_len + r + 1;

        double *v_root = (double *)malloc(sizeof(double) * (size_t)d);
        double *v_other = (double *)malloc(sizeof(double) * (size_t)d);
        double *x = (double *)malloc(sizeof(double) * (size_t)(prefix_len + n_self + 1));

        tree_query tq;
        tq.qv = qv; tq.k_ctx = k_ctx + (long)hk * d; tq.v_ctx = v_ctx + (long)hk * d;
        tq.cu = cu_chunk_lens; tq.n_chunks = n_chunks; tq.n_nodes = n_nodes; tq.d = d;
        tq.kv_stride = kv_stride; tq.score_scale = inv_sqrt_d / T;
        tq.node_scale = node_scale; tq.node_first = node_first; tq.node_count = node_count;
        tq.node_leaf = node_leaf; tq.bad = 0;
        const double A_root = tree_node_value(&tq, 0, v_root);
        if (tq.bad) bad = 1;

        /* non-context block: prefix and causal self tokens share one softmax (C.1) */
        for (long j = 0; j < prefix_len; ++j)
            x[j] = dot_fd(qv, k_prefix + j * kv_stride + (long)hk * d, d) * inv_sqrt_d;
        for (long j = 0; j < n_self; ++j)
            x[prefix_len + j] = dot_fd(qv, k_self + j * kv_stride + (long)hk * d, d) * inv_sqrt_d;
        const double A_other = logsumexp(x, prefix_len + n_self);
        for (int c = 0; c < d; ++c) v_other[c] = 0.0;
        for (long j = 0; j < prefix_len + n_self; ++j) {
            const double w = exp(x[j] - A_other);
            const float *vv = j < prefix_len ? v_prefix + j * kv_stride + (long)hk * d
                                             : v_self + (j - prefix_len) * kv_stride + (long)hk * d;
            for (int c = 0; c < d; ++c) v_other[c] += w * (double)vv[c];
        }

        const double two[2] = { A_root, A_other };
        const double Ltot = logsumexp(two, 2);
        const double w_root = A_root > -INFINITY ? exp(A_root - Ltot) : 0.0;
        const double w_other = exp(A_other - Ltot);
        double *o = out + p * d;
        for (int c = 0; c < d; ++c) o[c] = w_root * v_root[c] + w_other * v_other[c];
        if (lse) lse[p] = Ltot;
        free(v_root); free(v_other); free(x);
    }
    return bad ? -1 : 0;
}

/*
 * Section 2.2 "Pre-caching Contexts" with the shared prefix of Section 4.1.
 *
 * Context i is encoded as the sequence [prefix ; C_i] by ordinary causal
 * softmax attention (Section 2.3): row r of context i sees every prefix token
 * and tokens 0..r of its own context, scores q.k/sqrt(d); tokens of other
 * contexts are invisible.  No temperature, no scaling factor (they belong to
 * query-time attention only).
 *
 * q_ctx/k_ctx/v_ctx are the packed contexts [M, heads, d] with cu_chunk_lens.
 * pair_rows are packed row indices in [0, M).  Outputs as above.
 * Prefix rows themselves (plain causal attention over the prefix) are the case
 * prefix_len = 0, n_chunks = 1 of this same function.
 */
int ape_oracle_encode(int n_q_heads, int n_kv_heads, int d,
                      const float *k_prefix, const float *v_prefix, int prefix_len,
                      const float *q_ctx, const float *k_ctx, const float *v_ctx,
                      const int *cu_chunk_lens, int n_chunks,
                      const int *pair_rows, const int *pair_heads, long n_pairs,
                      double *out, double *lse)
{
    if (n_q_heads <= 0 || n_kv_heads <= 0 || d <= 0 || n_q_heads % n_kv_heads) return -1;
    if (prefix_len < 0 || n_chunks < 0) return -1;
    const int G = n_q_heads / n_kv_heads;
    const long M = n_chunks > 0 ? cu_chunk_lens[n_chunks] : 0;
    const long kv_stride = (long)n_kv_heads * d;
    const double inv_sqrt_d = 1.0 / sqrt((double)d);
    const int all = (pair_rows == NULL);
    if (all) n_pairs = M * n_q_heads;
    int bad = 0;

#pragma omp parallel for schedule(dynamic, 1)
    for (long p = 0; p < n_pairs; ++p) {
        const long r = all ? p / n_q_heads : pair_rows[p];
        const int h = all ? (int)(p % n_q_heads) : pair_heads[p];
        if (r < 0 || r >= M || h < 0 || h >= n_q_heads) { bad = 1; continue; }
        int i = 0;                                   /* context that owns packed row r */
        while (i + 1 < n_chunks && cu_chunk_lens[i + 1] <= r) ++i;
        const long c0 = cu_chunk_lens[i];
        const long n_own = r - c0 + 1;               /* causal inside the context */
        const int hk = h / G;
        const float *qv = q_ctx + (r * n_q_heads + h) * d;

        const long n = prefix_len + n_own;
        double *x = (double *)malloc(sizeof(double) * (size_t)n);
        for (long j = 0; j < prefix_len; ++j)
            x[j] = dot_fd(qv, k_prefix + j * kv_stride + (long)hk * d, d) * inv_sqrt_d;
        for (long j = 0; j < n_own; ++j)
            x[prefix_len + j] = dot_fd(qv, k_ctx + (c0 + j) * kv_stride + (long)hk * d, d) * inv_sqrt_d;
        const double L = logsumexp(x, n);
        double *o = out + p * d;
        for (int c = 0; c < d; ++c) o[c] = 0.0;
        for (long j = 0; j < n; ++j) {
            const double w = exp(x[j] - L);
            const float *vv = (j < prefix_len) ? v_prefix + j * kv_stride + (long)hk * d
                                               : v_ctx + (c0 + j - prefix_len) * kv_stride + (long)hk * d;
            for (int c = 0; c < d; ++c) o[c] += w * (double)vv[c];
        }
        if (lse) lse[p] = L;
        free(x);
    }
    return bad ? -1 : 0;
}

/*
 * Rotary position embedding with re-used positions (Section 1 "Re-using
 * Positions": every context is placed in the same range of positions;
 * Section 2.3 names relative position embeddings, the rotary one being what
 * the Llama-3 models of the paper use).
 *
 * x is packed [M, heads, d] over n_chunks segments given by cu_chunk_lens;
 * the token at index j of ANY segment has position position_offset + j.
 * Rotation of the published rotary embedding in its half-split pairing:
 * dims (c, c + d/2), c = 0 .. d/2-1, are one plane, turned by the angle
 * pos * base^(-2c/d):
 *   y[c]       = x[c] cos(a) - x[c + d/2] sin(a)
 *   y[c + d/2] = x[c + d/2] cos(a) + x[c] sin(a)
 * Everything in double.  Returns 0, or -1 on bad arguments (d must be even).
 */
int ape_oracle_rope(const float *x, int heads, int d,
                    const int *cu_chunk_lens, int n_chunks,
                    long position_offset, double base, double *y)
{
    if (heads <= 0 || d <= 0 || (d & 1) || n_chunks < 0 || !(base > 0.0)) return -1;
    const int half = d / 2;
    for (int i = 0; i < n_chunks; ++i) {
        if (cu_chunk_lens[i + 1] < cu_chunk_lens[i]) return -1;
        for (long t = cu_chunk_lens[i]; t < cu_chunk_lens[i + 1]; ++t) {
            const double pos = (double)(position_offset + (t - cu_chunk_lens[i]));
            for (int h = 0; h < heads; ++h) {
                const float *xr = x + (t * heads + h) * (long)d;
                double *yr = y + (t * heads + h) * (long)d;
                for (int c = 0; c < half; ++c) {
                    const double a = pos * pow(base, -2.0 * (double)c / (double)d);
                    const double cs = cos(a), sn = sin(a);
                    const double x1 = (double)xr[c], x2 = (double)xr[c + half];
                    yr[c] = x1 * cs - x2 * sn;
                    yr[c + half] = x2 * cs + x1 * sn;
                }
            }
        }
    }
    return 0;
}
