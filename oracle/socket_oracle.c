/*
 * SOCKET decode path: plain CPU oracle.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement
 * of what the GPU library must compute.  It is used by the tests, by the smoke
 * check and by the benchmark's CPU-baseline leg, and by nothing else.  It shares
 * no code, header, table or constant with the HIP library.
 *
 * Every function takes HOST pointers.  Floating-point inputs arrive as fp32
 * arrays holding the exact operand values (a bf16 operand is passed widened to
 * fp32, which is exact); all arithmetic is done in double.  Loops are written in
 * the order the paper states them: no blocking, no fusion.  The only concession
 * to run time is one `omp parallel for` over independent keys.
 *
 * Conventions (the paper leaves these open; both sides of the parity tests use
 * the same ones):
 *   - W is stored [d][L*P]; column l*P+i is hyperplane i of table l
 *     (the paper's W^(l) in R^{P x d}, row i).
 *   - sign(z) = +1 when z >= 0 (so -0.0 counts as +1), else -1.
 *   - bucket id: bit i of the id is 1 when plane i has sign +1; the corner c_r
 *     has c_{r,i} = +1 when bit i of r is set, else -1.
 *   - top-k order: larger score first, ties to the smaller index.
 *
 * Pins: every function here is pinned by tests/test_oracle_pins.py against
 * closed forms, limits, brute force, hand-worked cases and library routines; the one thing with no
 * pin is an end-to-end numeric value, for which the paper prints no worked
 * example ("parity unpinned" for end-to-end values only).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_OK 0
#define ORACLE_EINVAL -1
#define ORACLE_ENOMEM -2

/* ------------------------------------------------------------------------- *
 * Alg. 1 (PrecomputeKeyHashes): h = sign(W^(l) k_j), encoded as a bucket id.
 *   K      [n][d]      keys
 *   W      [d][L*P]    Gaussian hyperplanes
 *   codes  [n][L]      bucket ids in [0, 2^P)
 *   near_zero [n][L]   (nullable) set to 1 when some plane of that table has
 *                      |z| < zero_margin, i.e. the bit is numerically fragile.
 * ------------------------------------------------------------------------- */
int socket_oracle_hash_keys(const float *K, long n, int d, const float *W, int L,
                            int P, uint16_t *codes, uint8_t *near_zero,
                            double zero_margin) {
    if (!K || !W || !codes || n < 0 || d <= 0 || L <= 0 || P < 1 || P > 16)
        return ORACLE_EINVAL;
    const long LP = (long)L * P;
#pragma omp parallel for schedule(static)
    for (long j = 0; j < n; ++j) {
        for (int l = 0; l < L; ++l) {
            unsigned id = 0;
            int fragile = 0;
            for (int i = 0; i < P; ++i) {
                double z = 0.0;
                for (int c = 0; c < d; ++c)
                    z += (double)K[j * d + c] * (double)W[(long)c * LP + (long)l * P + i];
                if (z >= 0.0) id |= 1u << i;
                if (fabs(z) < zero_margin) fragile = 1;
            }
            codes[j * L + l] = (uint16_t)id;
            if (near_zero) near_zero[j * L + l] = (uint8_t)fragile;
        }
    }
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------- *
 * Alg. 2 (SoftBucketProbs): u = tanh(W^(l) q)/sqrt(d); logit(r) = u.c_r/tau;
 * p^(l)(.|q) = softmax over the R = 2^P corners.
 *   q [d],  W [d][L*P],  p [L][R] (output)
 * The softmax subtracts the largest logit before exponentiating, which does not
 * change its value.
 * ------------------------------------------------------------------------- */
int socket_oracle_soft_probs(const float *q, int d, const float *W, int L, int P,
                             double tau, double *p) {
    if (!q || !W || !p || d <= 0 || L <= 0 || P < 1 || P > 16 || !(tau > 0.0))
        return ORACLE_EINVAL;
    const long LP = (long)L * P;
    const long R = 1L << P;
    double u[16];
    for (int l = 0; l < L; ++l) {
        for (int i = 0; i < P; ++i) {
            double z = 0.0;
            for (int c = 0; c < d; ++c)
                z += (double)W[(long)c * LP + (long)l * P + i] * (double)q[c];
            u[i] = tanh(z) / sqrt((double)d);
        }
        double *pl = p + (long)l * R;
        double top = -INFINITY;
        for (long r = 0; r < R; ++r) {
            double dot = 0.0;
            for (int i = 0; i < P; ++i) dot += ((r >> i) & 1) ? u[i] : -u[i];
            pl[r] = dot / tau;
            if (pl[r] > top) top = pl[r];
        }
        double total = 0.0;
        for (long r = 0; r < R; ++r) {
            pl[r] = exp(pl[r] - top);
            total += pl[r];
        }
        for (long r = 0; r < R; ++r) pl[r] /= total;
    }
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------- *
 * Alg. 5 (SoftHashCollisionScores) with Eq. 3's soft score:
 *   w_j = nu_j * sum_l p^(l)(b_j^(l) | q)   for valid j,   -inf for masked j.
 * Grouped-query reading: a KV head serving G query heads scores each key by the
 * mean over those G queries of the soft score (G = 1 is exactly the paper).
 *   codes [n][L], p [G][L][R], vnorm [n] or NULL (nu = 1),
 *   mask [n] bytes or NULL; key j is valid when j < seq_len and (mask NULL or
 *   mask[j] != 0).   scores [n] (output)
 * ------------------------------------------------------------------------- */
int socket_oracle_score(const uint16_t *codes, long n, int L, int P, const double *p,
                        int G, const float *vnorm, const uint8_t *mask, long seq_len,
                        double *scores) {
    if (!codes || !p || !scores || n < 0 || L <= 0 || P < 1 || P > 16 || G <= 0)
        return ORACLE_EINVAL;
    const long R = 1L << P;
#pragma omp parallel for schedule(static)
    for (long j = 0; j < n; ++j) {
        if (j >= seq_len || (mask && !mask[j])) {
            scores[j] = -INFINITY;
            continue;
        }
        double mean = 0.0;
        for (int g = 0; g < G; ++g) {
            double s = 0.0;
            for (int l = 0; l < L; ++l)
                s += p[((long)g * L + l) * R + codes[j * L + l]];
            mean += s;
        }
        mean /= (double)G;
        scores[j] = (vnorm ? (double)vnorm[j] : 1.0) * mean;
    }
    return ORACLE_OK;
}

/* Eq. 3, left: hard collision count  s_hard = #{ l : b_j^(l) = b_q^(l) }. */
int socket_oracle_hard_score(const uint16_t *codes, long n, int L,
                             const uint16_t *qcodes, double *scores) {
    if (!codes || !qcodes || !scores || n < 0 || L <= 0) return ORACLE_EINVAL;
    for (long j = 0; j < n; ++j) {
        long hits = 0;
        for (int l = 0; l < L; ++l) hits += (codes[j * L + l] == qcodes[l]);
        scores[j] = (double)hits;
    }
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------- *
 * Alg. 3, TopK step: the k indices with the largest scores, by a full sort on
 * (score descending, index ascending).  Keys scored -inf are never selected.
 *   idx [k] output, unused tail = -1;  *n_selected = how many were written.
 * ------------------------------------------------------------------------- */
typedef struct {
    double s;
    int32_t j;
} scored_t;

static int by_score_then_index(const void *a, const void *b) {
    const scored_t *x = (const scored_t *)a, *y = (const scored_t *)b;
    if (x->s > y->s) return -1;
    if (x->s < y->s) return 1;
    return (x->j > y->j) - (x->j < y->j);
}

int socket_oracle_topk(const double *scores, long n, long k, int32_t *idx,
                       long *n_selected) {
    if (!scores || !idx || n < 0 || k < 0) return ORACLE_EINVAL;
    scored_t *all = (scored_t *)malloc((size_t)(n > 0 ? n : 1) * sizeof(scored_t));
    if (!all) return ORACLE_ENOMEM;
    long m = 0;
    for (long j = 0; j < n; ++j) {
        if (scores[j] == -INFINITY || scores[j] != scores[j]) continue;
        all[m].s = scores[j];
        all[m].j = (int32_t)j;
        ++m;
    }
    qsort(all, (size_t)m, sizeof(scored_t), by_score_then_index);
    long take = k < m ? k : m;
    for (long i = 0; i < take; ++i) idx[i] = all[i].j;
    for (long i = take; i < k; ++i) idx[i] = -1;
    if (n_selected) *n_selected = take;
    free(all);
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------- *
 * Eq. 2 (sparse attention over the index set S):
 *   alpha_i = exp(scale * k_i.q) / sum_{j in S} exp(scale * k_j.q),  y = sum alpha_i v_i
 * scale = 1 is the paper's definition (no 1/sqrt(d)).  Entries idx < 0 are
 * skipped; an empty set gives y = 0.  The largest logit is subtracted before
 * exponentiating, which leaves alpha unchanged.
 *   q [d], K [n][d], V [n][d], idx [k], y [d] output
 * ------------------------------------------------------------------------- */
int socket_oracle_sparse_decode(const float *q, const float *K, const float *V, long n,
                                int d, const int32_t *idx, long k, double scale,
                                double *y) {
    if (!q || !K || !V || !idx || !y || d <= 0 || k < 0) return ORACLE_EINVAL;
    for (int c = 0; c < d; ++c) y[c] = 0.0;
    double *t = (double *)malloc((size_t)(k > 0 ? k : 1) * sizeof(double));
    if (!t) return ORACLE_ENOMEM;
    double top = -INFINITY;
    for (long i = 0; i < k; ++i) {
        if (idx[i] < 0) continue;
        if (idx[i] >= n) {
            free(t);
            return ORACLE_EINVAL;
        }
        double dot = 0.0;
        for (int c = 0; c < d; ++c)
            dot += (double)K[(long)idx[i] * d + c] * (double)q[c];
        t[i] = scale * dot;
        if (t[i] > top) top = t[i];
    }
    double total = 0.0;
    for (long i = 0; i < k; ++i) {
        if (idx[i] < 0) continue;
        t[i] = exp(t[i] - top);
        total += t[i];
    }
    for (long i = 0; i < k; ++i) {
        if (idx[i] < 0) continue;
        double alpha = t[i] / total;
        for (int c = 0; c < d; ++c) y[c] += alpha * (double)V[(long)idx[i] * d + c];
    }
    free(t);
    return ORACLE_OK;
}

/* Eq. 1 (dense attention): Eq. 2 with S = all n tokens, written out directly. */
int socket_oracle_dense_decode(const float *q, const float *K, const float *V, long n,
                               int d, double scale, double *y) {
    if (!q || !K || !V || !y || d <= 0 || n < 0) return ORACLE_EINVAL;
    for (int c = 0; c < d; ++c) y[c] = 0.0;
    if (n == 0) return ORACLE_OK;
    double *t = (double *)malloc((size_t)n * sizeof(double));
    if (!t) return ORACLE_ENOMEM;
    double top = -INFINITY;
    for (long i = 0; i < n; ++i) {
        double dot = 0.0;
        for (int c = 0; c < d; ++c) dot += (double)K[i * d + c] * (double)q[c];
        t[i] = scale * dot;
        if (t[i] > top) top = t[i];
    }
    double total = 0.0;
    for (long i = 0; i < n; ++i) {
        t[i] = exp(t[i] - top);
        total += t[i];
    }
    for (long i = 0; i < n; ++i) {
        double a = t[i] / total;
        for (int c = 0; c < d; ++c) y[c] += a * (double)V[i * d + c];
    }
    free(t);
    return ORACLE_OK;
}

/* Alg. 1 also returns the value norms ||v_j||_2 that Alg. 3 ranks with. */
/* ------------------------------------------------------------------------- *
 * Sink and local-window tokens (Experiments, evaluation protocol: a small number
 * of sink and local window tokens is always kept).  The first n_sink and the
 * last n_window of the seq_len valid tokens get the score +inf, so that the TopK
 * step takes them first; they count towards k.  A masked token (-inf) stays
 * masked.  scores [n] is updated in place.
 * ------------------------------------------------------------------------- */
int socket_oracle_force_tokens(double *scores, long n, long seq_len, long n_sink, long n_window) {
    if (!scores || n < 0 || seq_len < 0 || seq_len > n || n_sink < 0 || n_window < 0) return ORACLE_EINVAL;
    for (long j = 0; j < seq_len; ++j) {
        int forced = (j < n_sink) || (j >= seq_len - n_window);
        if (forced && scores[j] != -INFINITY) scores[j] = INFINITY;
    }
    return ORACLE_OK;
}

int socket_oracle_value_norms(const float *V, long n, int d, float *vnorm) {
    if (!V || !vnorm || n < 0 || d <= 0) return ORACLE_EINVAL;
    for (long j = 0; j < n; ++j) {
        double s = 0.0;
        for (int c = 0; c < d; ++c) s += (double)V[j * d + c] * (double)V[j * d + c];
        vnorm[j] = (float)sqrt(s);
    }
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------- *
 * Ranking-quality metrics (appendix "Definitions of metrics", used for the
 * ranking-quality figure).  Index sets are arrays of distinct token positions.
 * ------------------------------------------------------------------------- */

/* how many entries of a[0..na) also occur in b[0..nb) (plain double loop) */
static long count_common(const int32_t *a, long na, const int32_t *b, long nb) {
    long common = 0;
    for (long i = 0; i < na; ++i)
        for (long j = 0; j < nb; ++j)
            if (a[i] == b[j]) {
                ++common;
                break;
            }
    return common;
}

/* Precision = |S_k intersect R| / k, S_k the k retrieved items, R the relevant ones. */
int socket_oracle_precision(const int32_t *retrieved, long k, const int32_t *relevant, long nrel,
                            double *out) {
    if (!retrieved || !relevant || !out || k <= 0 || nrel < 0) return ORACLE_EINVAL;
    *out = (double)count_common(retrieved, k, relevant, nrel) / (double)k;
    return ORACLE_OK;
}

/* Jaccard(A, B) = |A intersect B| / |A union B|; two empty sets give 1. */
int socket_oracle_jaccard(const int32_t *a, long na, const int32_t *b, long nb, double *out) {
    if (!out || na < 0 || nb < 0 || (na > 0 && !a) || (nb > 0 && !b)) return ORACLE_EINVAL;
    const long common = count_common(a, na, b, nb);
    const long uni = na + nb - common;
    *out = uni > 0 ? (double)common / (double)uni : 1.0;
    return ORACLE_OK;
}

static int descending(const void *x, const void *y) {
    const double a = *(const double *)x, b = *(const double *)y;
    return (a < b) - (a > b);
}

/* NDCG of a ranked list of length k: DCG = sum_{i=1..k} (2^{r_i} - 1) / log2(i + 1), r_i the
 * relevance of the item at rank i; IDCG is the DCG of the best list of length k that the n
 * candidate items allow, i.e. their k largest relevances in decreasing order; NDCG = DCG / IDCG.
 *   rel_ranked [k]  relevance of the retrieved items, best-ranked first
 *   rel_all    [n]  relevance of every candidate item, n >= k                              */
int socket_oracle_ndcg(const double *rel_ranked, long k, const double *rel_all, long n, double *out) {
    if (!rel_ranked || !rel_all || !out || k <= 0 || n < k) return ORACLE_EINVAL;
    double *sorted = (double *)malloc((size_t)n * sizeof(double));
    if (!sorted) return ORACLE_ENOMEM;
    memcpy(sorted, rel_all, (size_t)n * sizeof(double));
    qsort(sorted, (size_t)n, sizeof(double), descending);
    double dcg = 0.0, idcg = 0.0;
    for (long i = 1; i <= k; ++i) {
        const double discount = log2((double)i + 1.0);
        dcg += (pow(2.0, rel_ranked[i - 1]) - 1.0) / discount;
        idcg += (pow(2.0, sorted[i - 1]) - 1.0) / discount;
    }
    free(sorted);
    *out = idcg != 0.0 ? dcg / idcg : 0.0;
    return ORACLE_OK;
}
