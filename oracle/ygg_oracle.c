/*
 * ygg_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, fp64 CPU statement of what the tree-verification hot path of
 * Yggdrasil computes.  Only tests, the smoke check and the CPU-baseline leg of
 * the benchmark may call it; the GPU library never does, and the two share no
 * code.  Every function is the definition written out (nothing is blocked,
 * fused or re-ordered), so it can be checked against the paper by eye:
 *
 *   attention : a speculative token tree is verified in one parallel pass in
 *               which the attention mask encodes the tree's causal
 *               dependency (paper Sec. 2 "Source of Improvements", Sec. 4.2
 *               last paragraph): node i sees the confirmed prefix, its
 *               ancestors and itself.
 *   expand    : equal-growth drafting adds exactly W_draft leaves per draft
 *               step, chosen by largest path-wise gain with the drafter's
 *               generation probabilities as acceptance surrogates (Sec. 4.2
 *               "Draft Width Selection").  Reading used here: candidates are
 *               children of the previous depth's nodes, score = cumulative
 *               natural-log softmax probability along the path.
 *   accept    : the draft is accepted where it matches the verifier's own
 *               greedy token (Sec. 1; Sec. 5 "accept speculation management"),
 *               the verifier's token after the last accepted node is the bonus
 *               token (Sec. 4.1, text under Eq. 2), and the accepted nodes'
 *               K/V become part of the contiguous cache (Sec. 6, TokenTree).
 *
 * Pins (tests/test_oracle_*.py): per-path sequential attention, width-1 ==
 * causal attention via a library routine, closed forms (q = 0, constant V,
 * L = 0), split/merge identity, brute-force top-W and path enumeration,
 * hand-worked fixtures under tests/golden/.
 *
 * Element types: 0 = fp32, 1 = bf16 (stored as uint16, upper half of an fp32),
 * 2 = 8-bit E4M3 codes (K and V of the *_fp8kv variants and of the compaction
 * only; the paper does not fix the K/V precision, so this is a storage variant of
 * the same definition: a stored element stands for its per-kv-head scale times
 * the code's value).
 * All floating-point work is done in double.  Return value 0 = ok, negative =
 * invalid argument (see the checks at the top of each function).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_F32 = 0, ORC_BF16 = 1, ORC_FP8_E4M3 = 2 };

static size_t elem_bytes(int dtype) { return dtype == ORC_F32 ? 4u : dtype == ORC_BF16 ? 2u : 1u; }

/* 8-bit floating point, OCP E4M3: sign, 4 exponent bits (bias 7), 3 mantissa bits.
 * Exponent field 0 holds the subnormals m/8 * 2^-6; there are no infinities; the
 * all-ones exponent with all-ones mantissa is the only NaN; the largest finite
 * value is 1.75 * 2^8 = 448. */
static double fp8_e4m3_value(uint8_t code)
{
    const int sign = code >> 7, e = (code >> 3) & 15, m = code & 7;
    double v;
    if (e == 15 && m == 7)
        v = NAN;
    else if (e == 0)
        v = ldexp((double)m / 8.0, -6);
    else
        v = ldexp(1.0 + (double)m / 8.0, e - 7);
    return sign ? -v : v;
}

/* out[i] = value of code[i]; exposed so that tests can pin the table */
int ygg_oracle_fp8_e4m3_decode(const uint8_t *code, int64_t n, double *out)
{
    if (n < 0)
        return -1;
    for (int64_t i = 0; i < n; ++i)
        out[i] = fp8_e4m3_value(code[i]);
    return 0;
}

static double load_elem(const void *base, int dtype, int64_t idx)
{
    if (dtype == ORC_F32)
        return (double)((const float *)base)[idx];
    if (dtype == ORC_FP8_E4M3)
        return fp8_e4m3_value(((const uint8_t *)base)[idx]);
    uint16_t h = ((const uint16_t *)base)[idx];
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* parent[0] == -1 and 0 <= parent[i] < i for i > 0 */
static int tree_is_topological(const int32_t *parent, int32_t N)
{
    if (N < 1 || parent[0] != -1)
        return 0;
    for (int32_t i = 1; i < N; ++i)
        if (parent[i] < 0 || parent[i] >= i)
            return 0;
    return 1;
}

static int32_t node_depth(const int32_t *parent, int32_t i)
{
    int32_t d = 0;
    while (parent[i] >= 0) {
        i = parent[i];
        ++d;
    }
    return d;
}

/* ------------------------------------------------------------------------ *
 * Tree-masked verify attention, one output row.
 *
 * Layouts: q [B,N,Hq,Dh]; k_cache,v_cache [B,cap,Hkv,Dh] with rows
 * [0,seq_lens[b]) valid; k_tree,v_tree [B,N,Hkv,Dh]; parent_idx [B,N].
 * Query head h uses kv head h / (Hq/Hkv).
 *
 * Key set of node i:  J(i) = prefix rows 0..L-1  U  {i, parent[i], ..., root}.
 *   s_j = scale * <q_i, k_j>;  m = max_j s_j;  p_j = exp(s_j - m);
 *   l = sum_j p_j;  out = sum_j (p_j / l) v_j;  lse = m + ln l.
 * Keys outside J(i) are left out of every sum (never entered as -inf).
 *
 * probs (optional, length L + N): p_j / l for prefix key j at [j] and for tree
 * node t at [L + t]; exactly 0.0 for nodes outside J(i).
 * ------------------------------------------------------------------------ */
static int attention_row_core(int32_t B, int32_t N, int32_t Hq, int32_t Hkv, int32_t Dh,
                              int dtype /* of q */, int kv_dtype /* of K and V */,
                              const float *k_scale, const float *v_scale /* [Hkv] or NULL = 1 */,
                              double scale, int64_t cap,
                              const void *q, const void *k_cache, const void *v_cache,
                              const int32_t *seq_lens, const void *k_tree, const void *v_tree,
                              const int32_t *parent_idx,
                              int32_t b, int32_t i, int32_t h,
                              double *out_row /* [Dh] */, double *lse /* [1] or NULL */,
                              double *probs /* [L+N] or NULL */)
{
    if (B < 1 || N < 1 || Hq < 1 || Hkv < 1 || Dh < 1 || Hq % Hkv != 0)
        return -1;
    if (b < 0 || b >= B || i < 0 || i >= N || h < 0 || h >= Hq)
        return -2;
    const int32_t *parent = parent_idx + (int64_t)b * N;
    if (!tree_is_topological(parent, N))
        return -3;
    const int32_t L = seq_lens[b];
    if (L < 0 || (int64_t)L > cap)
        return -4;

    const int32_t G = Hq / Hkv;
    const int32_t hk = h / G;
    const int64_t q_off = (((int64_t)b * N + i) * Hq + h) * Dh;
    /* a stored K (V) element stands for k_scale[hk] (v_scale[hk]) times its decoded value */
    const double ks = k_scale ? (double)k_scale[hk] : 1.0;
    const double vs = v_scale ? (double)v_scale[hk] : 1.0;

    char *visible = (char *)calloc((size_t)N, 1);
    double *s = (double *)malloc(sizeof(double) * (size_t)(L + N));
    if (!visible || !s) {
        free(visible);
        free(s);
        return -5;
    }
    for (int32_t a = i; a >= 0; a = parent[a])
        visible[a] = 1;

    /* scores */
    double m = -INFINITY;
    for (int32_t j = 0; j < L; ++j) {
        const int64_t k_off = (((int64_t)b * cap + j) * Hkv + hk) * Dh;
        double dot = 0.0;
        for (int32_t d = 0; d < Dh; ++d)
            dot += load_elem(q, dtype, q_off + d) * (ks * load_elem(k_cache, kv_dtype, k_off + d));
        s[j] = scale * dot;
        if (s[j] > m)
            m = s[j];
    }
    for (int32_t t = 0; t < N; ++t) {
        if (!visible[t])
            continue;
        const int64_t k_off = (((int64_t)b * N + t) * Hkv + hk) * Dh;
        double dot = 0.0;
        for (int32_t d = 0; d < Dh; ++d)
            dot += load_elem(q, dtype, q_off + d) * (ks * load_elem(k_tree, kv_dtype, k_off + d));
        s[L + t] = scale * dot;
        if (s[L + t] > m)
            m = s[L + t];
    }

    /* softmax weights */
    double l = 0.0;
    for (int32_t j = 0; j < L; ++j) {
        s[j] = exp(s[j] - m);
        l += s[j];
    }
    for (int32_t t = 0; t < N; ++t) {
        if (!visible[t]) {
            s[L + t] = 0.0;
            continue;
        }
        s[L + t] = exp(s[L + t] - m);
        l += s[L + t];
    }

    /* weighted sum of values */
    for (int32_t d = 0; d < Dh; ++d)
        out_row[d] = 0.0;
    for (int32_t j = 0; j < L; ++j) {
        const int64_t v_off = (((int64_t)b * cap + j) * Hkv + hk) * Dh;
        const double w = s[j] / l;
        for (int32_t d = 0; d < Dh; ++d)
            out_row[d] += w * (vs * load_elem(v_cache, kv_dtype, v_off + d));
    }
    for (int32_t t = 0; t < N; ++t) {
        if (!visible[t])
            continue;
        const int64_t v_off = (((int64_t)b * N + t) * Hkv + hk) * Dh;
        const double w = s[L + t] / l;
        for (int32_t d = 0; d < Dh; ++d)
            out_row[d] += w * (vs * load_elem(v_tree, kv_dtype, v_off + d));
    }
    if (lse)
        *lse = m + log(l);
    if (probs)
        for (int32_t j = 0; j < L + N; ++j)
            probs[j] = s[j] / l;

    free(visible);
    free(s);
    return 0;
}

int ygg_oracle_attention_row(int32_t B, int32_t N, int32_t Hq, int32_t Hkv, int32_t Dh,
                             int dtype, double scale, int64_t cap,
                             const void *q, const void *k_cache, const void *v_cache,
                             const int32_t *seq_lens, const void *k_tree, const void *v_tree,
                             const int32_t *parent_idx,
                             int32_t b, int32_t i, int32_t h,
                             double *out_row /* [Dh] */, double *lse /* [1] or NULL */,
                             double *probs /* [L+N] or NULL */)
{
    return attention_row_core(B, N, Hq, Hkv, Dh, dtype, dtype, NULL, NULL, scale, cap, q, k_cache, v_cache,
                              seq_lens, k_tree, v_tree, parent_idx, b, i, h, out_row, lse, probs);
}

/* The same row with K and V stored as E4M3 codes (one byte per element, same layouts) and one
 * dequantisation factor per kv head: K = k_scale[hk] * value(code), V likewise.  q keeps `dtype`. */
int ygg_oracle_attention_row_fp8kv(int32_t B, int32_t N, int32_t Hq, int32_t Hkv, int32_t Dh,
                                   int dtype, double scale, int64_t cap,
                                   const void *q, const uint8_t *k_cache, const uint8_t *v_cache,
                                   const int32_t *seq_lens, const uint8_t *k_tree, const uint8_t *v_tree,
                                   const float *k_scale, const float *v_scale,
                                   const int32_t *parent_idx,
                                   int32_t b, int32_t i, int32_t h,
                                   double *out_row, double *lse, double *probs)
{
    if (!k_scale || !v_scale)
        return -6;
    return attention_row_core(B, N, Hq, Hkv, Dh, dtype, ORC_FP8_E4M3, k_scale, v_scale, scale, cap, q,
                              k_cache, v_cache, seq_lens, k_tree, v_tree, parent_idx, b, i, h, out_row, lse,
                              probs);
}

/* All rows: out [B,N,Hq,Dh] and lse [B,N,Hq] (lse may be NULL), in double. */
int ygg_oracle_tree_attention(int32_t B, int32_t N, int32_t Hq, int32_t Hkv, int32_t Dh,
                              int dtype, double scale, int64_t cap,
                              const void *q, const void *k_cache, const void *v_cache,
                              const int32_t *seq_lens, const void *k_tree, const void *v_tree,
                              const int32_t *parent_idx, double *out, double *lse)
{
    if (B < 1 || N < 1 || Hq < 1 || Hkv < 1 || Dh < 1 || Hq % Hkv != 0)
        return -1;
    int rc = 0;
    const int64_t rows = (int64_t)B * N * Hq;
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t r = 0; r < rows; ++r) {
        const int32_t h = (int32_t)(r % Hq);
        const int32_t i = (int32_t)((r / Hq) % N);
        const int32_t b = (int32_t)(r / ((int64_t)Hq * N));
        int e = ygg_oracle_attention_row(B, N, Hq, Hkv, Dh, dtype, scale, cap, q, k_cache, v_cache,
                                         seq_lens, k_tree, v_tree, parent_idx, b, i, h,
                                         out + r * Dh, lse ? lse + r : NULL, NULL);
        if (e != 0) {
#pragma omp critical
            rc = e;
        }
    }
    return rc;
}

int ygg_oracle_tree_attention_fp8kv(int32_t B, int32_t N, int32_t Hq, int32_t Hkv, int32_t Dh,
                                    int dtype, double scale, int64_t cap,
                                    const void *q, const uint8_t *k_cache, const uint8_t *v_cache,
                                    const int32_t *seq_lens, const uint8_t *k_tree, const uint8_t *v_tree,
                                    const float *k_scale, const float *v_scale,
                                    const int32_t *parent_idx, double *out, double *lse)
{
    if (B < 1 || N < 1 || Hq < 1 || Hkv < 1 || Dh < 1 || Hq % Hkv != 0)
        return -1;
    int rc = 0;
    const int64_t rows = (int64_t)B * N * Hq;
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t r = 0; r < rows; ++r) {
        const int32_t h = (int32_t)(r % Hq);
        const int32_t i = (int32_t)((r / Hq) % N);
        const int32_t b = (int32_t)(r / ((int64_t)Hq * N));
        int e = ygg_oracle_attention_row_fp8kv(B, N, Hq, Hkv, Dh, dtype, scale, cap, q, k_cache, v_cache,
                                               seq_lens, k_tree, v_tree, k_scale, v_scale, parent_idx, b, i, h,
                                               out + r * Dh, lse ? lse + r : NULL, NULL);
        if (e != 0) {
#pragma omp critical
            rc = e;
        }
    }
    return rc;
}

/* ------------------------------------------------------------------------ *
 * Equal-growth expansion.
 *
 * Depth-d nodes live at indices base_d = 1 + (d-1) W ... base_d + W - 1; the
 * root is node 0.  The frontier feeding depth d is the root (F = 1) for d = 1
 * and the W nodes of depth d-1 otherwise; logits row p belongs to frontier
 * node p.
 *
 *   lse_p  = ln sum_v exp(x[p,v])                      (max-subtracted)
 *   s(p,v) = cum[frontier p] + (x[p,v] - lse_p)
 * ------------------------------------------------------------------------ */
int ygg_oracle_expand_scores(int32_t F, int32_t V, const float *logits /* [F,V] */,
                             const float *cum_front /* [F] */, double *scores /* [F,V] */)
{
    if (F < 1 || V < 1)
        return -1;
    for (int32_t p = 0; p < F; ++p) {
        const float *x = logits + (int64_t)p * V;
        double mx = -INFINITY;
        for (int32_t v = 0; v < V; ++v)
            if ((double)x[v] > mx)
                mx = (double)x[v];
        double sum = 0.0;
        for (int32_t v = 0; v < V; ++v)
            sum += exp((double)x[v] - mx);
        const double lse = mx + log(sum);
        for (int32_t v = 0; v < V; ++v)
            scores[(int64_t)p * V + v] = (double)cum_front[p] + ((double)x[v] - lse);
    }
    return 0;
}

typedef struct {
    double s;
    int64_t flat; /* p * V + v */
} cand_t;

/* higher score first; equal scores: lower flat index first */
static int cand_cmp(const void *a, const void *b)
{
    const cand_t *x = (const cand_t *)a, *y = (const cand_t *)b;
    if (x->s > y->s)
        return -1;
    if (x->s < y->s)
        return 1;
    if (x->flat < y->flat)
        return -1;
    if (x->flat > y->flat)
        return 1;
    return 0;
}

/*
 * One draft step: all F*V candidates are scored and fully sorted; the first W
 * become the nodes of depth d in that order.  draft_logits [B,F,V];
 * parent_idx, token_ids, cum_logprob [B,N] with N = 1 + D*W (depth d-1 slots
 * are read, depth d slots are written; cum_logprob rounds the double score to
 * fp32 once).  margin[b] (optional) = score gap between the W-th and (W+1)-th
 * candidate (+inf if there is no (W+1)-th).
 */
int ygg_oracle_expand(int32_t B, int32_t D, int32_t W, int32_t V, int32_t d,
                      const float *draft_logits, int32_t *parent_idx, int32_t *token_ids,
                      float *cum_logprob, double *margin)
{
    if (B < 1 || D < 1 || W < 1 || V < 1 || d < 1 || d > D)
        return -1;
    const int32_t N = 1 + D * W;
    const int32_t F = d == 1 ? 1 : W;
    if ((int64_t)F * V < W)
        return -2; /* fewer candidates than slots */
    const int32_t base_prev = d == 1 ? 0 : 1 + (d - 2) * W;
    const int32_t base_new = 1 + (d - 1) * W;
    const int64_t C = (int64_t)F * V;

    double *scores = (double *)malloc(sizeof(double) * (size_t)C);
    cand_t *cand = (cand_t *)malloc(sizeof(cand_t) * (size_t)C);
    float *cum_front = (float *)malloc(sizeof(float) * (size_t)F);
    if (!scores || !cand || !cum_front) {
        free(scores);
        free(cand);
        free(cum_front);
        return -5;
    }
    for (int32_t b = 0; b < B; ++b) {
        for (int32_t p = 0; p < F; ++p)
            cum_front[p] = cum_logprob[(int64_t)b * N + base_prev + p];
        ygg_oracle_expand_scores(F, V, draft_logits + (int64_t)b * C, cum_front, scores);
        for (int64_t c = 0; c < C; ++c) {
            cand[c].s = scores[c];
            cand[c].flat = c;
        }
        qsort(cand, (size_t)C, sizeof(cand_t), cand_cmp);
        for (int32_t k = 0; k < W; ++k) {
            const int32_t p = (int32_t)(cand[k].flat / V);
            const int32_t v = (int32_t)(cand[k].flat % V);
            parent_idx[(int64_t)b * N + base_new + k] = base_prev + p;
            token_ids[(int64_t)b * N + base_new + k] = v;
            cum_logprob[(int64_t)b * N + base_new + k] = (float)cand[k].s;
        }
        if (margin)
            margin[b] = C > W ? cand[W - 1].s - cand[W].s : INFINITY;
    }
    free(scores);
    free(cand);
    free(cum_front);
    return 0;
}

/* ------------------------------------------------------------------------ *
 * Equal growth with free attachment (paper Sec. 4.2, "Draft Width Selection",
 * taken literally: every draft step grows exactly W leaves, and a leaf may hang
 * under any node of the partial tree, wherever the path-wise gain is largest).
 *
 * Reading: every node, once the drafter has run on it, offers its W most
 * probable tokens (larger logit first, equal logits: lower token first) as
 * candidate children, each scored cum[node] + log_softmax(row)[token].  The
 * pool holds every offer not yet taken.  Step t (1..D):
 *   1. the rows of draft_logits belong to the nodes added at step t-1 (the root
 *      for t = 1), in node order; their offers join the pool;
 *   2. the pool is ordered by (score descending, node*V + token ascending);
 *   3. the first W entries become nodes 1+(t-1)W .. tW in that order (parent =
 *      offering node, cum_logprob = score rounded to fp32) and leave the pool.
 * The pool is kept whole (nothing is ever dropped) and stays sorted.
 *
 * pool_score/pool_node/pool_token [B,pool_cap], pool_count [B]: in/out state;
 * step 1 ignores the incoming count.  margin[b] (optional) = score gap between
 * the W-th and (W+1)-th entry of the ordered pool (+inf if there is none).
 * ------------------------------------------------------------------------ */
typedef struct {
    float x;
    int32_t v;
} logit_t;

static int logit_cmp(const void *a, const void *b)
{
    const logit_t *x = (const logit_t *)a, *y = (const logit_t *)b;
    if (x->x > y->x)
        return -1;
    if (x->x < y->x)
        return 1;
    return x->v < y->v ? -1 : (x->v > y->v ? 1 : 0);
}

int ygg_oracle_attach(int32_t B, int32_t D, int32_t W, int32_t V, int32_t t,
                      const float *draft_logits, int32_t *parent_idx, int32_t *token_ids,
                      float *cum_logprob, double *pool_score, int32_t *pool_node,
                      int32_t *pool_token, int32_t *pool_count, int32_t pool_cap, double *margin)
{
    if (B < 1 || D < 1 || W < 1 || V < W || t < 1 || t > D || pool_cap < 1)
        return -1;
    const int32_t N = 1 + D * W;
    const int32_t F = t == 1 ? 1 : W;
    const int32_t base_prev = t == 1 ? 0 : 1 + (t - 2) * W;
    const int32_t base_new = 1 + (t - 1) * W;

    double *scores = (double *)malloc(sizeof(double) * (size_t)V);
    logit_t *order = (logit_t *)malloc(sizeof(logit_t) * (size_t)V);
    cand_t *pool = (cand_t *)malloc(sizeof(cand_t) * (size_t)pool_cap);
    if (!scores || !order || !pool) {
        free(scores);
        free(order);
        free(pool);
        return -5;
    }
    int rc = 0;
    for (int32_t b = 0; b < B && rc == 0; ++b) {
        int32_t n = t == 1 ? 0 : pool_count[b];
        if (n < 0 || n > pool_cap) {
            rc = -3;
            break;
        }
        for (int32_t i = 0; i < n; ++i) {
            pool[i].s = pool_score[(int64_t)b * pool_cap + i];
            pool[i].flat = (int64_t)pool_node[(int64_t)b * pool_cap + i] * V + pool_token[(int64_t)b * pool_cap + i];
        }
        for (int32_t p = 0; p < F; ++p) {
            const int32_t node = base_prev + p;
            const float *x = draft_logits + ((int64_t)b * F + p) * V;
            const float cum = cum_logprob[(int64_t)b * N + node];
            ygg_oracle_expand_scores(1, V, x, &cum, scores);
            for (int32_t v = 0; v < V; ++v) {
                order[v].x = x[v];
                order[v].v = v;
            }
            qsort(order, (size_t)V, sizeof(logit_t), logit_cmp);
            if (n + W > pool_cap) {
                rc = -7; /* the caller's pool is too small */
                break;
            }
            for (int32_t k = 0; k < W; ++k) {
                pool[n].s = scores[order[k].v];
                pool[n].flat = (int64_t)node * V + order[k].v;
                ++n;
            }
        }
        if (rc)
            break;
        qsort(pool, (size_t)n, sizeof(cand_t), cand_cmp);
        for (int32_t k = 0; k < W; ++k) {
            parent_idx[(int64_t)b * N + base_new + k] = (int32_t)(pool[k].flat / V);
            token_ids[(int64_t)b * N + base_new + k] = (int32_t)(pool[k].flat % V);
            cum_logprob[(int64_t)b * N + base_new + k] = (float)pool[k].s;
        }
        if (margin)
            margin[b] = n > W ? pool[W - 1].s - pool[W].s : INFINITY;
        for (int32_t i = W; i < n; ++i) {
            pool_score[(int64_t)b * pool_cap + i - W] = pool[i].s;
            pool_node[(int64_t)b * pool_cap + i - W] = (int32_t)(pool[i].flat / V);
            pool_token[(int64_t)b * pool_cap + i - W] = (int32_t)(pool[i].flat % V);
        }
        pool_count[b] = n - W;
    }
    free(scores);
    free(order);
    free(pool);
    return rc;
}

/* ------------------------------------------------------------------------ *
 * Verification-width pruning (paper Sec. 4.2, "Verification Width Pruning":
 * after drafting, a maximum-value subtree of the drafted tree is kept so that
 * W_verify tokens are verified; a bottom-up dynamic programme over the tree).
 *
 * ygg_oracle_subtree_dp: for a tree in topological order (parent[i] < i,
 * parent[0] = -1) with a value per node, best[k] (k = 1..N) = the largest total
 * value of a connected set of k nodes that contains the root, by the bottom-up
 * recurrence
 *     f_i[1] = value[i];  joining child c:  f_i[a+b] = max f_i[a] + f_c[b], b >= 0
 * (f_c[0] = 0: the child's subtree is left out).  keep[i] (optional) marks one
 * optimal set of `want` nodes.
 * ------------------------------------------------------------------------ */
int ygg_oracle_subtree_dp(int32_t N, const int32_t *parent, const double *value, int32_t want,
                          double *best /* [N+1], best[0] = 0 */, uint8_t *keep /* [N] or NULL */)
{
    if (N < 1 || parent[0] != -1 || want < 0 || want > N)
        return -1;
    for (int32_t i = 1; i < N; ++i)
        if (parent[i] < 0 || parent[i] >= i)
            return -4;
    /* f[i][k], k = 0..size_i: nodes of the subtree of i, i included when k >= 1 */
    int32_t *size = (int32_t *)calloc((size_t)N, sizeof(int32_t));
    double **f = (double **)calloc((size_t)N, sizeof(double *));
    /* choice[c][k] = how many nodes child c contributes when its parent's table (after joining c) holds k */
    int32_t **choice = (int32_t **)calloc((size_t)N, sizeof(int32_t *));
    if (!size || !f || !choice)
        return -5;
    for (int32_t i = 0; i < N; ++i) {
        f[i] = (double *)malloc(sizeof(double) * (size_t)(N + 1));
        choice[i] = (int32_t *)calloc((size_t)(N + 1), sizeof(int32_t));
        if (!f[i] || !choice[i])
            return -5;
        size[i] = 1;
        f[i][0] = 0.0;
        f[i][1] = value[i];
    }
    /* children join their parents in decreasing index order: every child is complete before it joins */
    for (int32_t c = N - 1; c >= 1; --c) {
        const int32_t p = parent[c];
        const int32_t sp = size[p], sc = size[c];
        double *g = (double *)malloc(sizeof(double) * (size_t)(sp + sc + 1));
        if (!g)
            return -5;
        for (int32_t k = 0; k <= sp + sc; ++k)
            g[k] = -INFINITY;
        g[0] = 0.0;
        for (int32_t a = 1; a <= sp; ++a)
            for (int32_t b = 0; b <= sc; ++b) {
                const double v = f[p][a] + f[c][b];
                if (v > g[a + b]) {
                    g[a + b] = v;
                    choice[c][a + b] = b;
                }
            }
        for (int32_t k = 0; k <= sp + sc; ++k)
            f[p][k] = g[k];
        size[p] = sp + sc;
        free(g);
    }
    best[0] = 0.0;
    for (int32_t k = 1; k <= N; ++k)
        best[k] = f[0][k];
    if (keep) {
        /* undo the joins in reverse order: the last child joined (lowest index) is split off first */
        int32_t *quota = (int32_t *)calloc((size_t)N, sizeof(int32_t));
        if (!quota)
            return -5;
        quota[0] = want;
        for (int32_t c = 1; c < N; ++c) {
            const int32_t p = parent[c];
            const int32_t b = quota[p] >= 1 ? choice[c][quota[p]] : 0;
            quota[c] = b;
            quota[p] -= b;
        }
        for (int32_t i = 0; i < N; ++i)
            keep[i] = quota[i] >= 1 ? 1 : 0;
        free(quota);
    }
    for (int32_t i = 0; i < N; ++i) {
        free(f[i]);
        free(choice[i]);
    }
    free(f);
    free(choice);
    free(size);
    return 0;
}

/*
 * Pruning of one batch of drafted trees to `w` nodes each.  The value of a node
 * is the probability that the whole path to it is accepted, with the drafter's
 * probabilities as surrogates: exp(cum_logprob[i]) (the root counts 1: the
 * bonus token).  The sum over a kept set estimates the accepted length.
 *   kept_nodes   [B,w]  original indices, ascending (still topological)
 *   new_parent   [B,w]  parent in the renumbered tree (-1 for the root)
 *   new_token    [B,w]
 *   expected_len [B]    sum of the kept values
 *   best_width   [B]    (optional, needs t_verifier [N+1] and t_draft) the n in 1..N maximising
 *                       best[n] / (t_draft + t_verifier[n])  (Eq. 3 with everything but W_verify
 *                       fixed; first maximum)
 */
int ygg_oracle_prune(int32_t B, int32_t N, int32_t w, const int32_t *parent_idx, const int32_t *token_ids,
                     const float *cum_logprob, const double *t_verifier, double t_draft,
                     int32_t *kept_nodes, int32_t *new_parent, int32_t *new_token, double *expected_len,
                     int32_t *best_width, double *best_curve /* [B,N+1] or NULL */)
{
    if (B < 1 || N < 1 || w < 1 || w > N)
        return -1;
    double *value = (double *)malloc(sizeof(double) * (size_t)N);
    double *best = (double *)malloc(sizeof(double) * (size_t)(N + 1));
    uint8_t *keep = (uint8_t *)malloc((size_t)N);
    int32_t *renum = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);
    if (!value || !best || !keep || !renum)
        return -5;
    int rc = 0;
    for (int32_t b = 0; b < B && rc == 0; ++b) {
        const int32_t *par = parent_idx + (int64_t)b * N;
        for (int32_t i = 0; i < N; ++i)
            value[i] = exp((double)cum_logprob[(int64_t)b * N + i]);
        rc = ygg_oracle_subtree_dp(N, par, value, w, best, keep);
        if (rc)
            break;
        int32_t k = 0;
        for (int32_t i = 0; i < N; ++i) {
            renum[i] = -1;
            if (keep[i]) {
                renum[i] = k;
                kept_nodes[(int64_t)b * w + k] = i;
                new_parent[(int64_t)b * w + k] = i == 0 ? -1 : renum[par[i]];
                new_token[(int64_t)b * w + k] = token_ids[(int64_t)b * N + i];
                ++k;
            }
        }
        if (k != w) {
            rc = -8;
            break;
        }
        expected_len[b] = best[w];
        if (best_curve)
            for (int32_t n = 0; n <= N; ++n)
                best_curve[(int64_t)b * (N + 1) + n] = best[n];
        if (best_width && t_verifier) {
            int32_t arg = 1;
            double top = -INFINITY;
            for (int32_t n = 1; n <= N; ++n) {
                const double obj = best[n] / (t_draft + t_verifier[n]);
                if (obj > top) {
                    top = obj;
                    arg = n;
                }
            }
            best_width[b] = arg;
        }
    }
    free(value);
    free(best);
    free(keep);
    free(renum);
    return rc;
}

/* ------------------------------------------------------------------------ *
 * Greedy acceptance and K/V compaction.
 *
 *   t*[i]    = first index of the maximum of target_logits[i,:]
 *              (or target_tokens[i] when the argmax is supplied)
 *   match[0] = 1;  match[i] = match[parent[i]] && token_ids[i] == t*[parent[i]]
 *   best     = matched node of greatest depth, lowest index among equals
 *   path     = root ... best;  accept_len = depth(best) + 1;  bonus = t*[best]
 *   every layer: cache[L_b + k] = tree[path[k]] for k < accept_len (K and V,
 *   all kv heads, raw bytes);  seq_lens[b] = L_b + accept_len.
 *
 * target_logits [B,N,V] fp32 or NULL; target_tokens [B,N] or NULL (exactly one
 * must be given); k_tree,v_tree [layers,B,N,Hkv,Dh]; k_cache,v_cache
 * [layers,B,cap,Hkv,Dh]; accept_path [B,path_cols], -1 padded; tstar_out
 * [B,N] optional.  Fails (-6) if the accepted path does not fit path_cols or
 * the cache (L_b + accept_len > cap).
 * ------------------------------------------------------------------------ */
int ygg_oracle_accept_compact(int32_t B, int32_t N, int32_t V, int32_t path_cols,
                              int32_t n_layers, int32_t Hkv, int32_t Dh, int dtype, int64_t cap,
                              const float *target_logits, const int32_t *target_tokens,
                              const int32_t *parent_idx, const int32_t *token_ids,
                              const void *k_tree, const void *v_tree,
                              void *k_cache, void *v_cache, int32_t *seq_lens,
                              int32_t *accept_len, int32_t *accept_path, int32_t *bonus_token,
                              int32_t *tstar_out)
{
    if (B < 1 || N < 1 || path_cols < 1 || n_layers < 0)
        return -1;
    if ((target_logits == NULL) == (target_tokens == NULL))
        return -2;
    if (target_logits && V < 1)
        return -2;

    int32_t *tstar = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);
    char *match = (char *)malloc((size_t)N);
    if (!tstar || !match) {
        free(tstar);
        free(match);
        return -5;
    }
    int rc = 0;
    const size_t row_bytes = (size_t)Hkv * (size_t)Dh * elem_bytes(dtype);

    for (int32_t b = 0; b < B && rc == 0; ++b) {
        const int32_t *parent = parent_idx + (int64_t)b * N;
        const int32_t *token = token_ids + (int64_t)b * N;
        if (!tree_is_topological(parent, N)) {
            rc = -3;
            break;
        }
        for (int32_t i = 0; i < N; ++i) {
            if (target_tokens) {
                tstar[i] = target_tokens[(int64_t)b * N + i];
            } else {
                const float *x = target_logits + ((int64_t)b * N + i) * V;
                int32_t arg = 0;
                for (int32_t v = 1; v < V; ++v)
                    if (x[v] > x[arg])
                        arg = v;
                tstar[i] = arg;
            }
            if (tstar_out)
                tstar_out[(int64_t)b * N + i] = tstar[i];
        }
        match[0] = 1;
        int32_t best = 0, best_depth = 0;
        for (int32_t i = 1; i < N; ++i) {
            match[i] = match[parent[i]] && token[i] == tstar[parent[i]];
            if (match[i]) {
                const int32_t dep = node_depth(parent, i);
                if (dep > best_depth) { /* strict: the lowest index wins ties */
                    best_depth = dep;
                    best = i;
                }
            }
        }
        const int32_t len = best_depth + 1;
        const int32_t L = seq_lens[b];
        if (len > path_cols || L < 0 || (int64_t)L + len > cap) {
            rc = -6;
            break;
        }
        for (int32_t k = 0; k < path_cols; ++k)
            accept_path[(int64_t)b * path_cols + k] = -1;
        for (int32_t a = best, k = len - 1; a >= 0; a = parent[a], --k)
            accept_path[(int64_t)b * path_cols + k] = a;
        accept_len[b] = len;
        bonus_token[b] = tstar[best];

        for (int32_t layer = 0; layer < n_layers; ++layer) {
            for (int32_t k = 0; k < len; ++k) {
                const int32_t node = accept_path[(int64_t)b * path_cols + k];
                const size_t src = (((size_t)layer * B + b) * N + node) * row_bytes;
                const size_t dst = (((size_t)layer * B + b) * (size_t)cap + (size_t)(L + k)) * row_bytes;
                memcpy((char *)k_cache + dst, (const char *)k_tree + src, row_bytes);
                memcpy((char *)v_cache + dst, (const char *)v_tree + src, row_bytes);
            }
        }
        seq_lens[b] = L + len;
    }
    free(tstar);
    free(match);
    return rc;
}

/* ------------------------------------------------------------------------ *
 * Check of the data-dependent part of the calling contract (the device calls
 * treat a violation as undefined behaviour).  flags[b] collects, per sequence:
 *   1  parent_idx[b][0] != -1, or some parent_idx[b][i] outside [0, i)
 *   2  seq_lens[b] outside [0, max_seq_len]
 *   4  some node deeper than `depth` (only judged when the parents are valid)
 *   8  some token_ids[b][i] outside [0, vocab)
 *  16  a NaN among logits[b][*][*]
 * Any of the arrays may be NULL: its checks are skipped.
 * ------------------------------------------------------------------------ */
int ygg_oracle_validate(int32_t B, int32_t N, int32_t depth, int32_t vocab, int32_t max_seq_len,
                        const int32_t *parent_idx, const int32_t *seq_lens, const int32_t *token_ids,
                        const float *logits, int32_t logit_rows, int32_t *flags)
{
    if (B < 1 || N < 1)
        return -1;
    int32_t *dep = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);
    if (!dep)
        return -5;
    for (int32_t b = 0; b < B; ++b) {
        int32_t f = 0;
        if (parent_idx) {
            const int32_t *par = parent_idx + (int64_t)b * N;
            int ok = par[0] == -1;
            for (int32_t i = 1; i < N; ++i)
                if (par[i] < 0 || par[i] >= i)
                    ok = 0;
            if (!ok) {
                f |= 1;
            } else {
                dep[0] = 0;
                for (int32_t i = 1; i < N; ++i) {
                    dep[i] = dep[par[i]] + 1;
                    if (dep[i] > depth)
                        f |= 4;
                }
            }
        }
        if (seq_lens && (seq_lens[b] < 0 || seq_lens[b] > max_seq_len))
            f |= 2;
        if (token_ids)
            for (int32_t i = 0; i < N; ++i)
                if (token_ids[(int64_t)b * N + i] < 0 || token_ids[(int64_t)b * N + i] >= vocab)
                    f |= 8;
        if (logits)
            for (int64_t e = 0; e < (int64_t)logit_rows * vocab; ++e)
                if (isnan(logits[(int64_t)b * logit_rows * vocab + e]))
                    f |= 16;
        flags[b] = f;
    }
    free(dep);
    return 0;
}

/* Number of threads the row-parallel loops above use (for the benchmark's CPU-baseline record; no arithmetic). */
int ygg_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
