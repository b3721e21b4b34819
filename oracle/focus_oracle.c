/*
 * focus_oracle.c -- TEST INFRASTRUCTURE, not part of the product path.
 *
 * A plain, slow, fp64 CPU statement of what the Focus inference attention
 * computes.  It materialises one dense boolean mask row per query and a masked
 * softmax over it; there is no tiling, no sorting, no online softmax.  It
 * shares no code with the HIP library and neither includes the other.
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 *
 * What it follows (paper: "Composing Sparse Attention via Learned Grouping"):
 *   - Sec. 2, first paragraph: softmax(Q K^T / sqrt(d)) V per head.
 *   - Sec. 2, Eq. 1 (form of the score: token vector dotted with centroids).
 *   - Sec. 2 "Efficiency at inference" and Sec. 3.6: every token keeps its
 *     top-k groups; a distant pair attends only when the two tokens share at
 *     least one group; nearby pairs always attend.
 *   - App. D, Eq. 3: the hard-assignment mask, causal AND (same group OR local).
 *   - Sec. 1: the softmax over the allowed pairs is exact (no renormalisation).
 *   - Sec. 2, Eq. 2: the soft-gated attention of training (focus_oracle_soft_rows).
 *
 * Readings taken where the paper is silent or the benchmark spec binds
 * differently (all restated in the design notes of the repository):
 *   - scores are raw dot products of the per-head query (or key) vector with
 *     per-KV-head centroids; no temperature, no normalisation before top-k;
 *   - canonical score precision: fp64, products added in index order t=0..d-1;
 *   - top-k ties: the smaller group index wins;
 *   - the local window holds exactly w keys including the query itself:
 *     i-w < j <= i (causal) or |i-j| < w (non-causal);
 *   - logit softcap: x = cap*tanh(scale*q.k/cap), applied before masking;
 *   - GQA: query head h uses KV head head_map[h] (default h / (Hq/Hkv)) for
 *     keys, values, key membership and centroids.
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC -o libfocus_oracle.so focus_oracle.c -lm
 * (no -ffast-math: the canonical score needs IEEE evaluation order).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int32_t B, Hq, Hkv, n, d;
    int32_t K, topk, window;
    int32_t causal;
    int32_t dtype;            /* 0 = fp32, 1 = bf16, 2 = IEEE binary16 (both as raw uint16 storage) */
    double scale;             /* 0 -> 1/sqrt(d) */
    double softcap;           /* 0 -> off */
    const int32_t *head_map;  /* [Hq] -> kv head, or NULL */
} oracle_params;

static double widen(const void *base, int dtype, int64_t idx)
{
    if (dtype == 0) {
        return (double)((const float *)base)[idx];
    } else if (dtype == 2) {
        /* IEEE 754 binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits */
        const uint16_t h = ((const uint16_t *)base)[idx];
        const int e = (h >> 10) & 31, m = h & 1023;
        double v;
        if (e == 0) v = ldexp((double)m, -24);
        else if (e == 31) v = m ? NAN : INFINITY;
        else v = ldexp((double)(1024 + m), e - 25);
        return (h >> 15) ? -v : v;
    } else {
        uint32_t bits = ((uint32_t)((const uint16_t *)base)[idx]) << 16;
        float f;
        memcpy(&f, &bits, 4);
        return (double)f;
    }
}

static int kv_of(const oracle_params *p, int h)
{
    if (p->head_map) return p->head_map[h];
    return h / (p->Hq / p->Hkv);
}

static int check_params(const oracle_params *p)
{
    if (!p) return -1;
    if (p->B < 1 || p->Hq < 1 || p->Hkv < 1 || p->n < 1 || p->d < 1) return -1;
    if (p->K < 1 || p->K > 32 || p->topk < 1 || p->topk > p->K) return -1;
    if (p->window < 1) return -1;
    if (p->dtype < 0 || p->dtype > 2) return -1;
    if (!p->head_map && (p->Hq % p->Hkv) != 0) return -1;
    if (p->head_map)
        for (int h = 0; h < p->Hq; ++h)
            if (p->head_map[h] < 0 || p->head_map[h] >= p->Hkv) return -1;
    return 0;
}

/* ------------------------------------------------------------------ scores
 * Eq. 1 (form): S[b,h,i,g] = sum_t x[b,h,i,t] * c[kv(h),g,t], fp64, t ascending.
 * x is q ([B,Hq,n,d], is_query=1) or k ([B,Hkv,n,d], is_query=0).
 * scores: [B,H,n,K].
 */
int focus_oracle_scores(const oracle_params *p, const void *x, int is_query,
                        const float *centroids, double *scores)
{
    if (check_params(p) || !x || !centroids || !scores) return -1;
    const int H = is_query ? p->Hq : p->Hkv;
    const int n = p->n, d = p->d, K = p->K;
    const int64_t rows = (int64_t)p->B * H * n;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        int h = (int)((r / n) % H);
        int hk = is_query ? kv_of(p, h) : h;
        for (int g = 0; g < K; ++g) {
            const float *c = centroids + ((int64_t)hk * K + g) * d;
            double acc = 0.0;
            for (int t = 0; t < d; ++t) {
                double prod = widen(x, p->dtype, r * d + t) * (double)c[t];
                acc = acc + prod;
            }
            scores[r * K + g] = acc;
        }
    }
    return 0;
}

/* -------------------------------------------------------------- membership
 * Sec. 2 "Efficiency at inference": keep the topk highest-scoring groups.
 * Group g is kept when fewer than topk groups beat it; g' beats g when its
 * score is larger, or equal with g' < g.  masks: [B,H,n] bit g set = member.
 * The paper says nothing of scores that are not numbers: a token with a NaN
 * among its K scores has no ranking and is given the first topk groups
 * (infinities are ordinary values of the order).
 */
static uint32_t topk_of_scores(const double *s, int K, int topk)
{
    for (int g = 0; g < K; ++g)
        if (isnan(s[g])) return (topk == 32) ? 0xffffffffu : ((1u << topk) - 1u);
    uint32_t m = 0;
    for (int g = 0; g < K; ++g) {
        int beaten_by = 0;
        for (int o = 0; o < K; ++o) {
            if (o == g) continue;
            if (s[o] > s[g] || (s[o] == s[g] && o < g)) ++beaten_by;
        }
        if (beaten_by < topk) m |= (1u << g);
    }
    return m;
}

int focus_oracle_topk_masks(const oracle_params *p, const double *scores, int H,
                            uint32_t *masks)
{
    if (check_params(p) || !scores || !masks) return -1;
    const int K = p->K;
    const int64_t rows = (int64_t)p->B * H * p->n;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        masks[r] = topk_of_scores(scores + r * K, K, p->topk);
    }
    return 0;
}

int focus_oracle_membership(const oracle_params *p, const void *x, int is_query,
                            const float *centroids, uint32_t *masks)
{
    if (check_params(p)) return -1;
    const int H = is_query ? p->Hq : p->Hkv;
    const int64_t rows = (int64_t)p->B * H * p->n;
    double *scores = (double *)malloc(sizeof(double) * (size_t)rows * p->K);
    if (!scores) return -2;
    int rc = focus_oracle_scores(p, x, is_query, centroids, scores);
    if (!rc) rc = focus_oracle_topk_masks(p, scores, H, masks);
    free(scores);
    return rc;
}

/* -------------------------------------------------------------- group lists
 * For every (b,h) and group g: how many tokens carry g, and their positions in
 * ascending order (the order a stable sort by group keeps; Sec. 2, App. D).
 * counts: [B,H,K]; lists: [B,H,topk*n], group g's list starts at the sum of the
 * counts of the groups before it.
 */
int focus_oracle_group_lists(const oracle_params *p, const uint32_t *masks, int H,
                             int32_t *counts, int32_t *lists)
{
    if (check_params(p) || !masks || !counts || !lists) return -1;
    const int n = p->n, K = p->K;
    for (int64_t bh = 0; bh < (int64_t)p->B * H; ++bh) {
        const uint32_t *m = masks + bh * n;
        int32_t *cnt = counts + bh * K;
        int32_t *lst = lists + bh * (int64_t)p->topk * n;
        int64_t w = 0;
        for (int g = 0; g < K; ++g) {
            int c = 0;
            for (int i = 0; i < n; ++i)
                if ((m[i] >> g) & 1u) { lst[w++] = i; ++c; }
            cnt[g] = c;
        }
    }
    return 0;
}

/* ------------------------------------------------------------ attention rows
 * For each requested query row (b,h,i):
 *   allowed(i,j) = (causal ? j <= i : 1) and (local(i,j) or mq[i] & mk[j] != 0)
 *   x_j = scale * q_i.k_j; softcap (if any); -inf where not allowed
 *   P = softmax(x); out = P V; lse = max + ln(sum exp(x - max));
 *   row_pairs = number of allowed j.
 * rows: nrows triples (b,h,i), or NULL meaning every row in (b,h,i) order.
 * out: [nrows,d] fp64; lse: [nrows] (nullable); row_pairs: [nrows] (nullable);
 * probs: [nrows,n] (nullable) the full probability rows.
 */
static int attn_rows_impl(const oracle_params *p, int pair_set, const void *q, const void *k,
                          const void *v, const uint32_t *mq, const uint32_t *mk,
                          int64_t nrows, const int32_t *rows, double *out,
                          double *lse, int64_t *row_pairs, double *probs)
{
    if (check_params(p) || !q || !k || !v || !mq || !mk || !out) return -1;
    const int n = p->n, d = p->d, Hq = p->Hq, Hkv = p->Hkv, w = p->window;
    const double scale = (p->scale != 0.0) ? p->scale : 1.0 / sqrt((double)d);
    const double cap = p->softcap;
    if (!rows && nrows != (int64_t)p->B * Hq * n) return -1;
    int bad = 0;
#pragma omp parallel
    {
        unsigned char *allowed = (unsigned char *)malloc((size_t)n);
        double *x = (double *)malloc(sizeof(double) * (size_t)n);
        double *qi = (double *)malloc(sizeof(double) * (size_t)d);
        if (!allowed || !x || !qi) {
#pragma omp atomic write
            bad = 1;
        } else {
#pragma omp for schedule(dynamic, 4)
            for (int64_t r = 0; r < nrows; ++r) {
                int b, h, i;
                if (rows) {
                    b = rows[3 * r]; h = rows[3 * r + 1]; i = rows[3 * r + 2];
                } else {
                    i = (int)(r % n); h = (int)((r / n) % Hq); b = (int)(r / ((int64_t)n * Hq));
                }
                if (b < 0 || b >= p->B || h < 0 || h >= Hq || i < 0 || i >= n) {
#pragma omp atomic write
                    bad = 1;
                    continue;
                }
                const int hk = kv_of(p, h);
                const int64_t qrow = ((int64_t)b * Hq + h) * n + i;
                const int64_t kbase = ((int64_t)b * Hkv + hk) * n;
                const uint32_t mi = mq[qrow];
                for (int t = 0; t < d; ++t) qi[t] = widen(q, p->dtype, qrow * d + t);
                /* the dense boolean mask row */
                int64_t npairs = 0;
                for (int j = 0; j < n; ++j) {
                    int in_range = p->causal ? (j <= i) : 1;
                    int local = p->causal ? (j > i - w && j <= i)
                                          : ((i - j < w) && (j - i < w));
                    int share = (mi & mk[kbase + j]) != 0;
                    int ok = (pair_set == 1) ? share                 /* set A: shares a group        */
                           : (pair_set == 2) ? (local && !share)     /* set B: local, no shared group */
                                             : (local || share);     /* the whole mask               */
                    allowed[j] = (unsigned char)(in_range && ok);
                    npairs += allowed[j];
                }
                if (npairs == 0) {                    /* only the sets A and B can leave a row empty */
                    for (int t = 0; t < d; ++t) out[r * d + t] = 0.0;
                    if (probs) for (int j = 0; j < n; ++j) probs[r * n + j] = 0.0;
                    if (lse) lse[r] = -INFINITY;
                    if (row_pairs) row_pairs[r] = 0;
                    continue;
                }
                /* logits and masked softmax */
                double mx = -INFINITY;
                for (int j = 0; j < n; ++j) {
                    if (!allowed[j]) { x[j] = -INFINITY; continue; }
                    double dot = 0.0;
                    for (int t = 0; t < d; ++t)
                        dot += qi[t] * widen(k, p->dtype, (kbase + j) * d + t);
                    double l = dot * scale;
                    if (cap > 0.0) l = cap * tanh(l / cap);
                    x[j] = l;
                    if (l > mx) mx = l;
                }
                double sum = 0.0;
                for (int j = 0; j < n; ++j) {
                    x[j] = allowed[j] ? exp(x[j] - mx) : 0.0;
                    sum += x[j];
                }
                double *o = out + r * d;
                for (int t = 0; t < d; ++t) o[t] = 0.0;
                for (int j = 0; j < n; ++j) {
                    if (!allowed[j]) continue;
                    double pj = x[j] / sum;
                    if (probs) probs[r * n + j] = pj;
                    for (int t = 0; t < d; ++t)
                        o[t] += pj * widen(v, p->dtype, (kbase + j) * d + t);
                }
                if (probs)
                    for (int j = 0; j < n; ++j)
                        if (!allowed[j]) probs[r * n + j] = 0.0;
                if (lse) lse[r] = mx + log(sum);
                if (row_pairs) row_pairs[r] = npairs;
            }
        }
        free(allowed); free(x); free(qi);
    }
    return bad ? -1 : 0;
}

/* Sec. 2 Eq. 2, the soft-gated attention of training: every causal pair is computed,
 *   s_ij = scale * (q_i . k_j) * gate_ij,
 *   gate_ij = 1                               for local pairs (i-w < j <= i),
 *           = sigmoid(lambda * g_i . g_j)     for the others,
 * followed by the exact softmax over j <= i and the product with V.  g [B,n,K] fp32 is the soft
 * assignment of every token of the layer (one per token, the same for all heads).  The equation is
 * taken literally: a gate of sigmoid(0) = 1/2 halves a logit, it does not remove the pair.
 * rows / out / lse as in attn_rows_impl; probs (nullable) [nrows,n].  causal only, no softcap. */
int focus_oracle_soft_rows(const oracle_params *p, double lambda, const float *g, const void *q,
                           const void *k, const void *v, int64_t nrows, const int32_t *rows,
                           double *out, double *lse, double *probs)
{
    if (check_params(p) || !g || !q || !k || !v || !out) return -1;
    if (!p->causal || p->softcap != 0.0) return -2;
    const int n = p->n, d = p->d, Hq = p->Hq, Hkv = p->Hkv, w = p->window, K = p->K;
    const double scale = (p->scale != 0.0) ? p->scale : 1.0 / sqrt((double)d);
    if (!rows && nrows != (int64_t)p->B * Hq * n) return -1;
    int bad = 0;
#pragma omp parallel
    {
        double *x = (double *)malloc(sizeof(double) * (size_t)n);
        double *qi = (double *)malloc(sizeof(double) * (size_t)d);
        if (!x || !qi) {
#pragma omp atomic write
            bad = 1;
        } else {
#pragma omp for schedule(dynamic, 4)
            for (int64_t r = 0; r < nrows; ++r) {
                int b, h, i;
                if (rows) {
                    b = rows[3 * r]; h = rows[3 * r + 1]; i = rows[3 * r + 2];
                } else {
                    i = (int)(r % n); h = (int)((r / n) % Hq); b = (int)(r / ((int64_t)n * Hq));
                }
                if (b < 0 || b >= p->B || h < 0 || h >= Hq || i < 0 || i >= n) {
#pragma omp atomic write
                    bad = 1;
                    continue;
                }
                const int hk = kv_of(p, h);
                const int64_t qrow = ((int64_t)b * Hq + h) * n + i;
                const int64_t kbase = ((int64_t)b * Hkv + hk) * n;
                const float *gi = g + ((int64_t)b * n + i) * K;
                for (int t = 0; t < d; ++t) qi[t] = widen(q, p->dtype, qrow * d + t);
                double mx = -INFINITY;
                for (int j = 0; j <= i; ++j) {
                    double dot = 0.0;
                    for (int t = 0; t < d; ++t)
                        dot += qi[t] * widen(k, p->dtype, (kbase + j) * d + t);
                    double gate = 1.0;
                    if (j <= i - w) {                         /* not local */
                        const float *gj = g + ((int64_t)b * n + j) * K;
                        double aff = 0.0;
                        for (int c = 0; c < K; ++c) aff += (double)gi[c] * (double)gj[c];
                        gate = 1.0 / (1.0 + exp(-lambda * aff));
                    }
                    x[j] = scale * dot * gate;
                    if (x[j] > mx) mx = x[j];
                }
                double sum = 0.0;
                for (int j = 0; j <= i; ++j) {
                    x[j] = exp(x[j] - mx);
                    sum += x[j];
                }
                double *o = out + r * d;
                for (int t = 0; t < d; ++t) o[t] = 0.0;
                if (probs)
                    for (int j = 0; j < n; ++j) probs[r * n + j] = 0.0;
                for (int j = 0; j <= i; ++j) {
                    double pj = x[j] / sum;
                    if (probs) probs[r * n + j] = pj;
                    for (int t = 0; t < d; ++t)
                        o[t] += pj * widen(v, p->dtype, (kbase + j) * d + t);
                }
                if (lse) lse[r] = mx + log(sum);
            }
        }
        free(x); free(qi);
    }
    return bad ? -1 : 0;
}

int focus_oracle_attn_rows(const oracle_params *p, const void *q, const void *k,
                           const void *v, const uint32_t *mq, const uint32_t *mk,
                           int64_t nrows, const int32_t *rows, double *out,
                           double *lse, int64_t *row_pairs, double *probs)
{
    return attn_rows_impl(p, 0, q, k, v, mq, mk, nrows, rows, out, lse, row_pairs, probs);
}

/* The paper's disjoint decomposition of the mask (App. D), with group sets in place of the
 * hard assignment g(i): pair_set 1 = A, causal pairs that share a group; pair_set 2 = B,
 * causal pairs inside the window that share none; 0 = their union, the whole mask.  Softmax
 * attention restricted to the set; a row with no pair in the set gives out = 0, lse = -inf. */
int focus_oracle_attn_rows_set(const oracle_params *p, int32_t pair_set, const void *q, const void *k,
                               const void *v, const uint32_t *mq, const uint32_t *mk,
                               int64_t nrows, const int32_t *rows, double *out,
                               double *lse, int64_t *row_pairs, double *probs)
{
    if (pair_set < 0 || pair_set > 2) return -1;
    return attn_rows_impl(p, pair_set, q, k, v, mq, mk, nrows, rows, out, lse, row_pairs, probs);
}

/* App. D "Merge": o = (e^{lA} oA + e^{lB} oB) / (e^{lA} + e^{lB}) per query row, and the
 * log-sum-exp of the union.  The larger of lA, lB is taken out of both exponentials first; a set
 * with lse = -inf weighs nothing. */
int focus_oracle_merge(int64_t nrows, int32_t d, const double *oa, const double *la,
                       const double *ob, const double *lb, double *out, double *lse)
{
    if (nrows < 0 || d < 1 || !oa || !la || !ob || !lb || !out) return -1;
    for (int64_t r = 0; r < nrows; ++r) {
        const double m = la[r] > lb[r] ? la[r] : lb[r];
        if (m == -INFINITY) {
            for (int t = 0; t < d; ++t) out[r * d + t] = 0.0;
            if (lse) lse[r] = -INFINITY;
            continue;
        }
        const double ea = exp(la[r] - m), eb = exp(lb[r] - m);
        for (int t = 0; t < d; ++t) out[r * d + t] = (ea * oa[r * d + t] + eb * ob[r * d + t]) / (ea + eb);
        if (lse) lse[r] = m + log(ea + eb);
    }
    return 0;
}

/* -------------------------------------------------------------- pair counts
 * Exact number of allowed pairs per (b,h) by inclusion-exclusion over the
 * shared-group sets, without visiting pairs (Sec. 3.6 cost model n^2/K is the
 * balanced special case).  With a_T(i) = [T subset of Gq(i)], b_T(j) likewise
 * for keys and cum_T the running count of b_T:
 *   L  = pairs inside the window (and the causal range)
 *   S  = sum over non-empty T, |T| <= topk, of (-1)^(|T|+1) sum_i a_T(i) * #b_T in range(i)
 *   SL = the same restricted to the window
 *   allowed = L + S - SL
 * A pair sharing m >= 1 groups is counted sum_t (-1)^(t+1) C(m,t) = 1 time.
 * group_pairs[b,h,g] = number of in-range pairs whose query and key both carry g.
 */
static uint32_t next_combination(uint32_t x)
{
    uint32_t c = x & (0u - x);
    uint32_t r = x + c;
    if (r == 0) return 0;
    return (((r ^ x) >> 2) / c) | r;
}

int focus_oracle_pair_counts(const oracle_params *p, const uint32_t *mq,
                             const uint32_t *mk, uint64_t *allowed_pairs,
                             uint64_t *group_pairs)
{
    if (check_params(p) || !mq || !mk || !allowed_pairs) return -1;
    const int n = p->n, K = p->K, w = p->window, Hq = p->Hq, Hkv = p->Hkv;
    /* number of subsets to visit */
    double nsub = 0.0, c = 1.0;
    for (int t = 1; t <= p->topk; ++t) { c = c * (K - t + 1) / t; nsub += c; }
    if (nsub > 2.0e6) return -3;
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t bh = 0; bh < (int64_t)p->B * Hq; ++bh) {
        const int b = (int)(bh / Hq), h = (int)(bh % Hq), hk = kv_of(p, h);
        const uint32_t *mi = mq + bh * n;
        const uint32_t *mj = mk + ((int64_t)b * Hkv + hk) * n;
        int64_t *cum = (int64_t *)malloc(sizeof(int64_t) * ((size_t)n + 1));
        if (!cum) {
#pragma omp atomic write
            bad = 1;
            continue;
        }
        int64_t L = 0, S = 0, SL = 0;
        for (int i = 0; i < n; ++i) {
            int lo = i - w + 1; if (lo < 0) lo = 0;
            int hi = p->causal ? i : (i + w - 1 < n - 1 ? i + w - 1 : n - 1);
            L += hi - lo + 1;
        }
        for (int t = 1; t <= p->topk; ++t) {
            const int64_t sign = (t & 1) ? 1 : -1;
            uint32_t T = (t == 32) ? 0xffffffffu : ((1u << t) - 1u);
            const uint64_t limit = (K == 32) ? 0x100000000ull : (1ull << K);
            while (T != 0 && (uint64_t)T < limit) {
                cum[0] = 0;
                for (int j = 0; j < n; ++j) cum[j + 1] = cum[j] + ((mj[j] & T) == T);
                int64_t sT = 0, wT = 0;
                for (int i = 0; i < n; ++i) {
                    if ((mi[i] & T) != T) continue;
                    int ulo = 0;
                    int uhi = p->causal ? i : n - 1;
                    int lo = i - w + 1; if (lo < 0) lo = 0;
                    int hi = p->causal ? i : (i + w - 1 < n - 1 ? i + w - 1 : n - 1);
                    sT += cum[uhi + 1] - cum[ulo];
                    wT += cum[hi + 1] - cum[lo];
                }
                S += sign * sT;
                SL += sign * wT;
                if (t == 1 && group_pairs) {
                    int g = 0; while (!((T >> g) & 1u)) ++g;
                    group_pairs[bh * K + g] = (uint64_t)sT;
                }
                if (t == 32) break;
                T = next_combination(T);
            }
        }
        allowed_pairs[bh] = (uint64_t)(L + S - SL);
        free(cum);
    }
    return bad ? -2 : 0;
}

int focus_oracle_num_threads(void)
{
    int nt = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        nt = omp_get_num_threads();
    }
#endif
    return nt;
}

/* ------------------------------------------------------------------ router
 * The paper's router (Sec. 2, Eq. 1 and the Sinkhorn recipe below it): one soft
 * assignment per token of a layer, shared by every head and by the query and
 * key roles:
 *     z_i = W_g^T h_i            (h_i: hidden state, dm values; W_g: dm x dg)
 *     S[i,g] = z_i . C[g]        (C: K x dg centroids)
 *     no normalisation (iters = 0):   g_i = S[i,:] / tau
 *     Sinkhorn (iters = N > 0):       Q = exp(S / tau); N times { every column divided by its
 *                                     sum over the tokens of the sequence, then every row divided
 *                                     by its sum over the groups };  g_i = Q[i,:]
 * Inference keeps the topk largest entries of g_i (Sec. 2 "Efficiency at inference").
 *
 * Readings (restated in the design notes): fp64 throughout; the projection is the
 * plain inner product, its products added one by one in index order t = 0 .. dm-1;
 * S adds over the dg components in index order; before the exponential the largest score of the sequence is subtracted
 * (the first column step divides any common factor out again, so the recipe is
 * unchanged, and exp cannot overflow); Sinkhorn runs per batch element over its
 * n tokens; ties in the top-k go to the smaller group index.
 *
 * hidden [B,n,dm] in dtype (0 fp32, 1 bf16 bits, 2 binary16 bits); wg [dm,dg] fp32; cent [K,dg] fp32.
 * z_out [B,n,dg], g_out [B,n,K] nullable fp64; masks [B,n] (bit g = member).
 */
int focus_oracle_route(int32_t B, int32_t n, int32_t dm, int32_t dg, int32_t K, int32_t topk,
                       int32_t dtype, const void *hidden, const float *wg, const float *cent,
                       double tau, int32_t iters, double *z_out, double *g_out, uint32_t *masks)
{
    if (B < 1 || n < 1 || dm < 1 || dg < 1 || K < 1 || K > 32 || topk < 1 || topk > K) return -1;
    if (!(tau > 0.0) || iters < 0 || !hidden || !wg || !cent || !masks) return -1;
    if (dtype < 0 || dtype > 2) return -1;
    if (dg > 256) return -1;                    /* z of one token lives in a 256-entry array below */
    double *Q = (double *)malloc(sizeof(double) * (size_t)n * K);
    if (!Q) return -2;
    for (int b = 0; b < B; ++b) {
        /* projection and scores */
#pragma omp parallel for schedule(static)
        for (int i = 0; i < n; ++i) {
            double z[256];
            const int64_t row = ((int64_t)b * n + i) * dm;
            for (int j = 0; j < dg; ++j) {
                double acc = 0.0;
                for (int t = 0; t < dm; ++t) acc += widen(hidden, dtype, row + t) * (double)wg[(int64_t)t * dg + j];
                z[j] = acc;
                if (z_out) z_out[((int64_t)b * n + i) * dg + j] = acc;
            }
            for (int g = 0; g < K; ++g) {
                double s = 0.0;
                for (int j = 0; j < dg; ++j) s += z[j] * (double)cent[(int64_t)g * dg + j];
                Q[(int64_t)i * K + g] = s;
            }
        }
        if (iters == 0) {
            for (int64_t e = 0; e < (int64_t)n * K; ++e) Q[e] = Q[e] / tau;
        } else {
            double smax = Q[0];
            for (int64_t e = 1; e < (int64_t)n * K; ++e) if (Q[e] > smax) smax = Q[e];
            for (int64_t e = 0; e < (int64_t)n * K; ++e) Q[e] = exp((Q[e] - smax) / tau);
            for (int it = 0; it < iters; ++it) {
                for (int g = 0; g < K; ++g) {            /* columns: sum over the tokens */
                    double cs = 0.0;
                    for (int i = 0; i < n; ++i) cs += Q[(int64_t)i * K + g];
                    for (int i = 0; i < n; ++i) Q[(int64_t)i * K + g] /= cs;
                }
                for (int i = 0; i < n; ++i) {            /* rows: sum over the groups */
                    double rs = 0.0;
                    for (int g = 0; g < K; ++g) rs += Q[(int64_t)i * K + g];
                    for (int g = 0; g < K; ++g) Q[(int64_t)i * K + g] /= rs;
                }
            }
        }
        for (int i = 0; i < n; ++i) {
            const double *s = Q + (int64_t)i * K;
            masks[(int64_t)b * n + i] = topk_of_scores(s, K, topk);
            if (g_out) for (int g = 0; g < K; ++g) g_out[((int64_t)b * n + i) * K + g] = s[g];
        }
    }
    free(Q);
    return 0;
}

/* Attention rows when membership is one mask per TOKEN (the paper's per-layer
 * assignment): the same mask serves every query head and every KV head. */
int focus_oracle_broadcast_masks(const oracle_params *p, const uint32_t *token_masks,
                                 uint32_t *mq, uint32_t *mk)
{
    if (check_params(p) || !token_masks || !mq || !mk) return -1;
    for (int b = 0; b < p->B; ++b) {
        for (int h = 0; h < p->Hq; ++h)
            memcpy(mq + ((int64_t)b * p->Hq + h) * p->n, token_masks + (int64_t)b * p->n, sizeof(uint32_t) * (size_t)p->n);
        for (int h = 0; h < p->Hkv; ++h)
            memcpy(mk + ((int64_t)b * p->Hkv + h) * p->n, token_masks + (int64_t)b * p->n, sizeof(uint32_t) * (size_t)p->n);
    }
    return 0;
}
