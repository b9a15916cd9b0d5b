/*
 * AhaKV eviction path -- float64 CPU oracle.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what
 * the eviction path computes, written from the paper's definitions.  It is
 * used by the tests, by the smoke check and by the benchmark's CPU-baseline
 * leg.  The GPU library never links, loads or calls it, and it shares no
 * code with the GPU library.
 *
 * Everything is double precision; tensors are dense, row-major, with the
 * layouts stated at each function.  Token positions are 0-indexed: query
 * row i sees keys 0..i, that is c_i = i + 1 keys.
 *
 * Parallelism: OpenMP over (batch, head) only.  No blocking, no fusion, no
 * reordering of the sums beyond what the definitions state.
 *
 * Readings of the paper that this file takes (the paper is silent, garbled
 * or ambiguous there) are marked "READING" below.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define AHA_ORACLE_SCALE_FIXED 0
#define AHA_ORACLE_SCALE_ADAPTIVE 1

/* ------------------------------------------------------------------------
 * Adaptive scale (Sec. 4.2, the closed form that follows from setting the
 * expected row entropy  log i - lambda^2 d / 2  equal to  log k):
 *     lambda = sqrt( 2 log(i / k) / d ).
 * READING: i is the number of keys the row normalises over (c), k is the
 * total budget B, log is natural.  For c <= k the logarithm is not positive;
 * it is clamped at 0, and the result is floored at `floor_` (a negative
 * `floor_` means the standard softmax scale 1/sqrt(d)).
 * ---------------------------------------------------------------------- */
double aha_oracle_lambda(int64_t c, int64_t k, int64_t d, double floor_)
{
    double lg = log((double)c / (double)k);
    if (lg < 0.0) lg = 0.0;
    double lam = sqrt(2.0 * lg / (double)d);
    double fl = (floor_ < 0.0) ? 1.0 / sqrt((double)d) : floor_;
    return lam > fl ? lam : fl;
}

static double row_scale(int scale_mode, double fixed_scale, double lambda_floor,
                        int64_t c, int64_t budget, int64_t d)
{
    if (scale_mode == AHA_ORACLE_SCALE_FIXED) return fixed_scale;
    return aha_oracle_lambda(c, budget, d, lambda_floor);
}

/* ------------------------------------------------------------------------
 * One row of the (step-gain) softmax attention matrix (Eq. for a_{i,j} in
 * Sec. 4.1 with the causal mask; SG-softmax of Sec. 4.2).
 * READING: SG-softmax(x; lambda)_j = exp(lambda x_j) / sum_j' exp(lambda x_j'),
 * applied to the RAW dot products w_ij = Q_i . K_j, i.e. lambda takes the place
 * of 1/sqrt(d).
 *
 * q: [d]; K: [>= c, d]; p: [c] receives the probabilities over keys 0..c-1.
 * ---------------------------------------------------------------------- */
static void softmax_row(const double *q, const double *K, int64_t c, int64_t d,
                        double scale, double *p)
{
    double m = -INFINITY;
    for (int64_t j = 0; j < c; ++j) {
        double w = 0.0;
        for (int64_t t = 0; t < d; ++t) w += q[t] * K[j * d + t];
        p[j] = scale * w;
        if (p[j] > m) m = p[j];
    }
    double z = 0.0;
    for (int64_t j = 0; j < c; ++j) {
        p[j] = exp(p[j] - m);
        z += p[j];
    }
    for (int64_t j = 0; j < c; ++j) p[j] /= z;
}

/* ------------------------------------------------------------------------
 * The observed rows of the attention matrix, written out (for tests that
 * check row sums, entropies, or compare against a library softmax).
 *
 * Q: [batch, n_q_heads, n, d], K: [batch, n_kv_heads, n, d]
 * P: [batch, n_q_heads, window, n]; row ii is query position n-window+ii,
 *    entries beyond the causal limit are 0.
 * ---------------------------------------------------------------------- */
void aha_oracle_attention_rows(const double *Q, const double *K,
                               int64_t batch, int64_t n_q_heads, int64_t n_kv_heads,
                               int64_t n, int64_t d, int64_t window, int64_t budget,
                               int scale_mode, double fixed_scale, double lambda_floor,
                               double *P)
{
    int64_t G = n_q_heads / n_kv_heads;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int64_t b = 0; b < batch; ++b) {
        for (int64_t hq = 0; hq < n_q_heads; ++hq) {
            int64_t hk = hq / G;
            const double *Kh = K + ((b * n_kv_heads + hk) * n) * d;
            for (int64_t ii = 0; ii < window; ++ii) {
                int64_t i = n - window + ii;
                int64_t c = i + 1;
                const double *q = Q + (((b * n_q_heads + hq) * n) + i) * d;
                double *p = P + (((b * n_q_heads + hq) * window) + ii) * n;
                double s = row_scale(scale_mode, fixed_scale, lambda_floor, c, budget, d);
                softmax_row(q, Kh, c, d, s, p);
                for (int64_t j = c; j < n; ++j) p[j] = 0.0;
            }
        }
    }
}

/* ------------------------------------------------------------------------
 * Value prior (Sec. 4.3):  nu_j = ||V_j||^2,  gamma = Avgpool(nu),
 * gamma_bar = gamma / max(gamma).
 * READING: the pool is 1-D over tokens, stride 1, odd width `pool`, output
 * length n; at the edges the mean is taken over the taps that fall inside
 * [0, n) (so a constant nu gives a constant gamma).  The maximum is per
 * (batch, KV head) over all n tokens.
 * READING: a head whose value rows are all zero has max(gamma) = 0 and the
 * quotient is undefined; the prior then carries no information and
 * gamma_bar is 1 everywhere (the scores stay unrefined).
 *
 * V: [batch, n_kv_heads, n, d];  gamma_bar: [batch, n_kv_heads, n]
 * ---------------------------------------------------------------------- */
void aha_oracle_value_prior(const double *V, int64_t batch, int64_t n_kv_heads,
                            int64_t n, int64_t d, int64_t pool, double *gamma_bar)
{
    int64_t half = (pool - 1) / 2;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int64_t b = 0; b < batch; ++b) {
        for (int64_t h = 0; h < n_kv_heads; ++h) {
            const double *Vh = V + ((b * n_kv_heads + h) * n) * d;
            double *g = gamma_bar + (b * n_kv_heads + h) * n;
            double *nu = (double *)malloc(sizeof(double) * (size_t)n);
            for (int64_t j = 0; j < n; ++j) {
                double s = 0.0;
                for (int64_t t = 0; t < d; ++t) s += Vh[j * d + t] * Vh[j * d + t];
                nu[j] = s;
            }
            double gmax = -INFINITY;
            for (int64_t j = 0; j < n; ++j) {
                int64_t lo = j - half < 0 ? 0 : j - half;
                int64_t hi = j + half > n - 1 ? n - 1 : j + half;
                double s = 0.0;
                for (int64_t t = lo; t <= hi; ++t) s += nu[t];
                g[j] = s / (double)(hi - lo + 1);
                if (g[j] > gmax) gmax = g[j];
            }
            for (int64_t j = 0; j < n; ++j) g[j] = gmax > 0.0 ? g[j] / gmax : 1.0;
            free(nu);
        }
    }
}

/* ------------------------------------------------------------------------
 * Prefill eviction scores (Sec. 4.1 Recent Accumulation; Alg. 1, Prefill):
 *     S_j = sum over the last `window` query rows i of p_ij,
 * p being the (SG-)softmax row of softmax_row().  With value_prior != 0 the
 * result is multiplied by gamma_bar (Sec. 4.3, last equation).
 * READING: exactly `window` rows are summed (positions n-window .. n-1).
 * READING (grouped-query attention, which the paper does not mention): the
 * score of a KV head is the SUM over the query heads that share it.
 * window == n, fixed scale 1/sqrt(d), value_prior == 0 is the plain
 * accumulated attention score of Sec. 4.1 (the H2O score).
 *
 * Q: [batch, n_q_heads, n, d]; K, V: [batch, n_kv_heads, n, d]
 * S: [batch, n_kv_heads, n]
 * ---------------------------------------------------------------------- */
void aha_oracle_prefill_scores(const double *Q, const double *K, const double *V,
                               int64_t batch, int64_t n_q_heads, int64_t n_kv_heads,
                               int64_t n, int64_t d, int64_t window, int64_t budget,
                               int scale_mode, double fixed_scale, double lambda_floor,
                               int value_prior, int64_t pool, double *S)
{
    int64_t G = n_q_heads / n_kv_heads;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int64_t b = 0; b < batch; ++b) {
        for (int64_t hk = 0; hk < n_kv_heads; ++hk) {
            const double *Kh = K + ((b * n_kv_heads + hk) * n) * d;
            double *Sh = S + (b * n_kv_heads + hk) * n;
            double *p = (double *)malloc(sizeof(double) * (size_t)n);
            for (int64_t j = 0; j < n; ++j) Sh[j] = 0.0;
            for (int64_t g = 0; g < G; ++g) {
                int64_t hq = hk * G + g;
                for (int64_t i = n - window; i < n; ++i) {
                    int64_t c = i + 1;
                    const double *q = Q + (((b * n_q_heads + hq) * n) + i) * d;
                    double s = row_scale(scale_mode, fixed_scale, lambda_floor, c, budget, d);
                    softmax_row(q, Kh, c, d, s, p);
                    for (int64_t j = 0; j < c; ++j) Sh[j] += p[j];
                }
            }
            free(p);
        }
    }
    if (value_prior) {
        double *gb = (double *)malloc(sizeof(double) * (size_t)(batch * n_kv_heads * n));
        aha_oracle_value_prior(V, batch, n_kv_heads, n, d, pool, gb);
        for (int64_t t = 0; t < batch * n_kv_heads * n; ++t) S[t] *= gb[t];
        free(gb);
    }
}

/* ------------------------------------------------------------------------
 * Prefill eviction scores accumulated over GIVEN query rows (Limitations: the
 * choice of the constant number of accumulators is not unique - instead of
 * the most recent rows one may select the same number of rows by a Top-k
 * strategy).
 * READING: the paper names no criterion for that Top-k; the rows are the
 * caller's choice, `window` positions per (batch, query head), and everything
 * else is the method unchanged: row at position i attends keys j <= i with the
 * scale of a row over c = i + 1 keys, the rows' probabilities are summed per
 * key (over the group's heads too), the value prior refines the sum.  With
 * rows = n-window .. n-1 for every head this is aha_oracle_prefill_scores.
 *
 * rows: [batch, n_q_heads, window] int32 positions in [0, n); other layouts
 * as aha_oracle_prefill_scores.
 * ---------------------------------------------------------------------- */
void aha_oracle_prefill_scores_rows(const double *Q, const double *K, const double *V,
                                    const int32_t *rows,
                                    int64_t batch, int64_t n_q_heads, int64_t n_kv_heads,
                                    int64_t n, int64_t d, int64_t window, int64_t budget,
                                    int scale_mode, double fixed_scale, double lambda_floor,
                                    int value_prior, int64_t pool, double *S)
{
    int64_t G = n_q_heads / n_kv_heads;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int64_t b = 0; b < batch; ++b) {
        for (int64_t hk = 0; hk < n_kv_heads; ++hk) {
            const double *Kh = K + ((b * n_kv_heads + hk) * n) * d;
            double *Sh = S + (b * n_kv_heads + hk) * n;
            double *p = (double *)malloc(sizeof(double) * (size_t)n);
            for (int64_t j = 0; j < n; ++j) Sh[j] = 0.0;
            for (int64_t g = 0; g < G; ++g) {
                int64_t hq = hk * G + g;
                for (int64_t ii = 0; ii < window; ++ii) {
                    int64_t i = rows[(b * n_q_heads + hq) * window + ii];
                    int64_t c = i + 1;
                    const double *q = Q + (((b * n_q_heads + hq) * n) + i) * d;
                    double s = row_scale(scale_mode, fixed_scale, lambda_floor, c, budget, d);
                    softmax_row(q, Kh, c, d, s, p);
                    for (int64_t j = 0; j < c; ++j) Sh[j] += p[j];
                }
            }
            free(p);
        }
    }
    if (value_prior) {
        double *gb = (double *)malloc(sizeof(double) * (size_t)(batch * n_kv_heads * n));
        aha_oracle_value_prior(V, batch, n_kv_heads, n, d, pool, gb);
        for (int64_t t = 0; t < batch * n_kv_heads * n; ++t) S[t] *= gb[t];
        free(gb);
    }
}

/* ------------------------------------------------------------------------
 * Row normalisers of the observed rows, as an attention forward pass emits
 * them (App. on compatibility with FlashAttention: the score is computed
 * beside a forward pass that keeps, per query row, the logarithm of the
 * softmax denominator):
 *     lse_i = log sum_{j <= i} exp(s w_ij),   natural logarithm, s = the row's scale.
 *
 * Q: [batch, n_q_heads, n, d], K: [batch, n_kv_heads, n, d]
 * lse: [batch, n_q_heads, window]; entry ii is query position n-window+ii.
 * ---------------------------------------------------------------------- */
void aha_oracle_row_lse(const double *Q, const double *K,
                        int64_t batch, int64_t n_q_heads, int64_t n_kv_heads,
                        int64_t n, int64_t d, int64_t window, int64_t budget,
                        int scale_mode, double fixed_scale, double lambda_floor,
                        double *lse)
{
    int64_t G = n_q_heads / n_kv_heads;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int64_t b = 0; b < batch; ++b) {
        for (int64_t hq = 0; hq < n_q_heads; ++hq) {
            const double *Kh = K + ((b * n_kv_heads + hq / G) * n) * d;
            for (int64_t ii = 0; ii < window; ++ii) {
                int64_t i = n - window + ii, c = i + 1;
                const double *q = Q + (((b * n_q_heads + hq) * n) + i) * d;
                double s = row_scale(scale_mode, fixed_scale, lambda_floor, c, budget, d);
                double m = -INFINITY;
                for (int64_t j = 0; j < c; ++j) {
                    double w = 0.0;
                    for (int64_t t = 0; t < d; ++t) w += q[t] * Kh[j * d + t];
                    if (s * w > m) m = s * w;
                }
                double z = 0.0;
                for (int64_t j = 0; j < c; ++j) {
                    double w = 0.0;
                    for (int64_t t = 0; t < d; ++t) w += q[t] * Kh[j * d + t];
                    z += exp(s * w - m);
                }
                lse[((b * n_q_heads + hq) * window) + ii] = m + log(z);
            }
        }
    }
}

/* ------------------------------------------------------------------------
 * Attention output of the observed rows (the self-attention that the score is
 * computed beside, App. on compatibility with FlashAttention; Alg. 1 Prefill
 * builds both from the same logits A = Q K^T / sqrt(d)):
 *     O_i = sum_{j <= i} softmax_j(Q_i . K_j / sqrt(d)) V_j
 * for the last `window` query positions, always with the standard scale.
 *
 * Q: [batch, n_q_heads, n, d]; K, V: [batch, n_kv_heads, n, d]
 * O: [batch, n_q_heads, window, d]; row ii is query position n-window+ii.
 * ---------------------------------------------------------------------- */
void aha_oracle_window_attention(const double *Q, const double *K, const double *V,
                                 int64_t batch, int64_t n_q_heads, int64_t n_kv_heads,
                                 int64_t n, int64_t d, int64_t window, double *O)
{
    int64_t G = n_q_heads / n_kv_heads;
    double s = 1.0 / sqrt((double)d);
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int64_t b = 0; b < batch; ++b) {
        for (int64_t hq = 0; hq < n_q_heads; ++hq) {
            const double *Kh = K + ((b * n_kv_heads + hq / G) * n) * d;
            const double *Vh = V + ((b * n_kv_heads + hq / G) * n) * d;
            double *p = (double *)malloc(sizeof(double) * (size_t)n);
            for (int64_t ii = 0; ii < window; ++ii) {
                int64_t i = n - window + ii, c = i + 1;
                const double *q = Q + (((b * n_q_heads + hq) * n) + i) * d;
                double *o = O + (((b * n_q_heads + hq) * window) + ii) * d;
                softmax_row(q, Kh, c, d, s, p);
                for (int64_t t = 0; t < d; ++t) o[t] = 0.0;
                for (int64_t j = 0; j < c; ++j)
                    for (int64_t t = 0; t < d; ++t) o[t] += p[j] * Vh[j * d + t];
            }
            free(p);
        }
    }
}

/* ------------------------------------------------------------------------
 * Information entropy of the observed rows (Sec. 4.2, the definition
 * H_i = - sum_j a_ij log a_ij over the keys j <= i the row attends to,
 * natural logarithm; a term with a_ij = 0 contributes 0), under the scale the
 * row uses.  With the standard scale its expectation on Gaussian logits is
 * log i - d/2 (scaled by 1/sqrt(d): log i - 1/2), with the adaptive scale it
 * is log k by construction.
 *
 * Q: [batch, n_q_heads, n, d], K: [batch, n_kv_heads, n, d]
 * H: [batch, n_q_heads, window]; entry ii is query position n-window+ii.
 * ---------------------------------------------------------------------- */
void aha_oracle_row_entropy(const double *Q, const double *K,
                            int64_t batch, int64_t n_q_heads, int64_t n_kv_heads,
                            int64_t n, int64_t d, int64_t window, int64_t budget,
                            int scale_mode, double fixed_scale, double lambda_floor,
                            double *H)
{
    int64_t G = n_q_heads / n_kv_heads;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int64_t b = 0; b < batch; ++b) {
        for (int64_t hq = 0; hq < n_q_heads; ++hq) {
            const double *Kh = K + ((b * n_kv_heads + hq / G) * n) * d;
            double *p = (double *)malloc(sizeof(double) * (size_t)n);
            for (int64_t ii = 0; ii < window; ++ii) {
                int64_t i = n - window + ii, c = i + 1;
                const double *q = Q + (((b * n_q_heads + hq) * n) + i) * d;
                double s = row_scale(scale_mode, fixed_scale, lambda_floor, c, budget, d);
                softmax_row(q, Kh, c, d, s, p);
                double h = 0.0;
                for (int64_t j = 0; j < c; ++j)
                    if (p[j] > 0.0) h -= p[j] * log(p[j]);
                H[((b * n_q_heads + hq) * window) + ii] = h;
            }
            free(p);
        }
    }
}

/* ------------------------------------------------------------------------
 * Prefill eviction scores from given row normalisers: the same sum as
 * aha_oracle_prefill_scores, with p_ij = exp(s w_ij - lse_i) taken from the
 * caller's lse instead of normalising the row here.  With the lse of
 * aha_oracle_row_lse for the same scale the two functions agree up to
 * rounding; a different lse scales row i's contribution by exp(true - given).
 *
 * lse: [batch, n_q_heads, window]; other layouts as aha_oracle_prefill_scores.
 * ---------------------------------------------------------------------- */
void aha_oracle_prefill_scores_lse(const double *Q, const double *K, const double *V,
                                   const double *lse,
                                   int64_t batch, int64_t n_q_heads, int64_t n_kv_heads,
                                   int64_t n, int64_t d, int64_t window, int64_t budget,
                                   int scale_mode, double fixed_scale, double lambda_floor,
                                   int value_prior, int64_t pool, double *S)
{
    int64_t G = n_q_heads / n_kv_heads;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int64_t b = 0; b < batch; ++b) {
        for (int64_t hk = 0; hk < n_kv_heads; ++hk) {
            const double *Kh = K + ((b * n_kv_heads + hk) * n) * d;
            double *Sh = S + (b * n_kv_heads + hk) * n;
            for (int64_t j = 0; j < n; ++j) Sh[j] = 0.0;
            for (int64_t g = 0; g < G; ++g) {
                int64_t hq = hk * G + g;
                for (int64_t ii = 0; ii < window; ++ii) {
                    int64_t i = n - window + ii, c = i + 1;
                    const double *q = Q + (((b * n_q_heads + hq) * n) + i) * d;
                    double s = row_scale(scale_mode, fixed_scale, lambda_floor, c, budget, d);
                    double L = lse[((b * n_q_heads + hq) * window) + ii];
                    for (int64_t j = 0; j < c; ++j) {
                        double w = 0.0;
                        for (int64_t t = 0; t < d; ++t) w += q[t] * Kh[j * d + t];
                        Sh[j] += exp(s * w - L);
                    }
                }
            }
        }
    }
    if (value_prior) {
        double *gb = (double *)malloc(sizeof(double) * (size_t)(batch * n_kv_heads * n));
        aha_oracle_value_prior(V, batch, n_kv_heads, n, d, pool, gb);
        for (int64_t t = 0; t < batch * n_kv_heads * n; ++t) S[t] *= gb[t];
        free(gb);
    }
}

/* ------------------------------------------------------------------------
 * Selection (Alg. 1: recent set, TopK, union).
 * READING: the TopK runs over the non-recent tokens j < n - recent, on the
 * value-refined score; ties go to the lower index; the result is the union
 * with the `recent` last tokens, in ascending token order, exactly `budget`
 * entries (budget = recent + selected, budget <= n).
 *
 * scores: [problems, n];  idx: [problems, budget] (int32)
 * ---------------------------------------------------------------------- */
typedef struct { double s; int64_t j; } scored_t;

static int cmp_scored(const void *a, const void *b)
{
    const scored_t *x = (const scored_t *)a, *y = (const scored_t *)b;
    if (x->s > y->s) return -1;
    if (x->s < y->s) return 1;
    return (x->j > y->j) - (x->j < y->j);
}

static int cmp_i64(const void *a, const void *b)
{
    int64_t x = *(const int64_t *)a, y = *(const int64_t *)b;
    return (x > y) - (x < y);
}

void aha_oracle_select_topk(const double *scores, int64_t problems, int64_t n,
                            int64_t budget, int64_t recent, int32_t *idx)
{
    int64_t n_cand = n - recent;
    int64_t n_sel = budget - recent;
#pragma omp parallel for schedule(dynamic)
    for (int64_t pr = 0; pr < problems; ++pr) {
        const double *s = scores + pr * n;
        int32_t *out = idx + pr * budget;
        scored_t *c = (scored_t *)malloc(sizeof(scored_t) * (size_t)(n_cand > 0 ? n_cand : 1));
        int64_t *keep = (int64_t *)malloc(sizeof(int64_t) * (size_t)(budget > 0 ? budget : 1));
        for (int64_t j = 0; j < n_cand; ++j) { c[j].s = s[j]; c[j].j = j; }
        qsort(c, (size_t)n_cand, sizeof(scored_t), cmp_scored);
        for (int64_t t = 0; t < n_sel; ++t) keep[t] = c[t].j;
        qsort(keep, (size_t)n_sel, sizeof(int64_t), cmp_i64);
        for (int64_t t = 0; t < recent; ++t) keep[n_sel + t] = n_cand + t;
        for (int64_t t = 0; t < budget; ++t) out[t] = (int32_t)keep[t];
        free(c);
        free(keep);
    }
}

/* ------------------------------------------------------------------------
 * Selection with attention-sink tokens (related work: the static policy that
 * keeps the first few tokens and the most recent ones, because the beginning
 * of the sequence matters for the whole generation).
 * READING: as a mode of the method's selection, the first `sink` tokens are
 * always retained like the `recent` last ones, and the remaining
 * budget - sink - recent places go to the highest scores among the tokens in
 * between (ties to the lower index).  sink = 0 is aha_oracle_select_topk;
 * budget = sink + recent is the static policy, which looks at no score.
 * Requires sink + recent <= budget <= n.
 *
 * scores: [problems, n];  idx: [problems, budget] (int32), ascending
 * ---------------------------------------------------------------------- */
void aha_oracle_select_topk_sink(const double *scores, int64_t problems, int64_t n,
                                 int64_t budget, int64_t recent, int64_t sink, int32_t *idx)
{
    int64_t first_recent = n - recent;
    int64_t n_mid = first_recent - sink;          /* candidates sink .. n-recent-1 */
    int64_t n_sel = budget - recent - sink;
#pragma omp parallel for schedule(dynamic)
    for (int64_t pr = 0; pr < problems; ++pr) {
        const double *s = scores + pr * n;
        int32_t *out = idx + pr * budget;
        scored_t *c = (scored_t *)malloc(sizeof(scored_t) * (size_t)(n_mid > 0 ? n_mid : 1));
        int64_t *keep = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n_sel > 0 ? n_sel : 1));
        for (int64_t j = 0; j < n_mid; ++j) { c[j].s = s[sink + j]; c[j].j = sink + j; }
        qsort(c, (size_t)(n_mid > 0 ? n_mid : 0), sizeof(scored_t), cmp_scored);
        for (int64_t t = 0; t < n_sel; ++t) keep[t] = c[t].j;
        qsort(keep, (size_t)n_sel, sizeof(int64_t), cmp_i64);
        for (int64_t t = 0; t < sink; ++t) out[t] = (int32_t)t;
        for (int64_t t = 0; t < n_sel; ++t) out[sink + t] = (int32_t)keep[t];
        for (int64_t t = 0; t < recent; ++t) out[sink + n_sel + t] = (int32_t)(first_recent + t);
        free(c);
        free(keep);
    }
}

/* ------------------------------------------------------------------------
 * Smoothing of the eviction scores before the selection (caption of the
 * method's overview figure: pooling is applied to the refined scores so that
 * the retained text is not sparsified excessively).
 * READING: a 1-D average pool over tokens with the conventions of the value
 * prior's pool (stride 1, odd width, mean over the taps inside [0, n)),
 * applied to the refined scores of ALL n tokens; the pooled values only rank
 * the candidates, the running scores F_0 stay the unpooled ones (Alg. 1).
 *
 * scores: [problems, n];  pooled: [problems, n]
 * ---------------------------------------------------------------------- */
void aha_oracle_pool_scores(const double *scores, int64_t problems, int64_t n,
                            int64_t pool, double *pooled)
{
    int64_t half = (pool - 1) / 2;
#pragma omp parallel for schedule(dynamic)
    for (int64_t pr = 0; pr < problems; ++pr) {
        const double *s = scores + pr * n;
        double *o = pooled + pr * n;
        for (int64_t j = 0; j < n; ++j) {
            int64_t lo = j - half < 0 ? 0 : j - half;
            int64_t hi = j + half > n - 1 ? n - 1 : j + half;
            double acc = 0.0;
            for (int64_t t = lo; t <= hi; ++t) acc += s[t];
            o[j] = acc / (double)(hi - lo + 1);
        }
    }
}

/* ------------------------------------------------------------------------
 * Compaction (Alg. 1, Generation: K_S, V_S; F_0 = refined prefill score).
 * Slot s of the compact cache holds token idx[s]; slot `budget` is left free
 * for the first generated token (free_slot = budget).  Slots >= budget get
 * position -1, score 0 and zero rows.
 *
 * K, V: [problems, n, d]; scores: [problems, n]; idx: [problems, budget]
 * Kc, Vc: [problems, slots, d]; Fc: [problems, slots]; pos: [problems, slots]
 * free_slot: [problems]
 * ---------------------------------------------------------------------- */
void aha_oracle_compact_kv(const double *K, const double *V, const double *scores,
                           const int32_t *idx, int64_t problems, int64_t n, int64_t d,
                           int64_t budget, int64_t slots,
                           double *Kc, double *Vc, double *Fc, int32_t *pos,
                           int32_t *free_slot)
{
    for (int64_t pr = 0; pr < problems; ++pr) {
        for (int64_t s = 0; s < slots; ++s) {
            double *kc = Kc + (pr * slots + s) * d;
            double *vc = Vc + (pr * slots + s) * d;
            if (s < budget) {
                int64_t j = idx[pr * budget + s];
                memcpy(kc, K + (pr * n + j) * d, sizeof(double) * (size_t)d);
                memcpy(vc, V + (pr * n + j) * d, sizeof(double) * (size_t)d);
                Fc[pr * slots + s] = scores[pr * n + j];
                pos[pr * slots + s] = (int32_t)j;
            } else {
                memset(kc, 0, sizeof(double) * (size_t)d);
                memset(vc, 0, sizeof(double) * (size_t)d);
                Fc[pr * slots + s] = 0.0;
                pos[pr * slots + s] = -1;
            }
        }
        free_slot[pr] = (int32_t)budget;
    }
}

/* ------------------------------------------------------------------------
 * One generation step with running eviction (Alg. 1, Generation loop body),
 * for every (batch, KV head):
 *   1. the new key/value row goes into the free slot, with score 0 and
 *      position logical_pos - 1 (logical_pos = tokens seen so far, the new
 *      one included);
 *   2. raw dots w_s = q . Kc[s] over the budget + 1 live slots;
 *   3. attention output  o = sum_s softmax_s(w_s / sqrt(d)) Vc[s];
 *   4. running score  F[s] += sum over the group's query heads of
 *      softmax_s(scale * w_s), scale as in the prefill with c = logical_pos;
 *   5. the `recent` slots with the largest positions are protected; among
 *      the others the one with the smallest F is evicted (ties: the one with
 *      the highest position), its position becomes -1 and it is the next
 *      free slot.
 * READING: the new token starts from score 0; the generation step adds the
 * unrefined probabilities (no value prior), as the algorithm is printed;
 * the output uses 1/sqrt(d) and the score uses the adaptive scale, both from
 * the same raw dots; c for the adaptive scale is the number of tokens seen,
 * not the cache length.
 * Only slots 0..budget are live; any slots beyond are ignored.
 *
 * q: [problems, G, d]; k_new, v_new: [problems, d]
 * Kc, Vc: [problems, slots, d]; Fc, pos: [problems, slots]; free_slot: [problems]
 * out: [problems, G, d]
 * ---------------------------------------------------------------------- */
void aha_oracle_decode_step_ext(const double *q, const double *k_new, const double *v_new,
                                int64_t problems, int64_t G, int64_t d,
                                int64_t budget, int64_t recent, int64_t slots,
                                int64_t logical_pos,
                                int scale_mode, double fixed_scale, double lambda_floor,
                                int64_t sink, int value_prior,
                                double *Kc, double *Vc, double *Fc, int32_t *pos,
                                int32_t *free_slot, double *out);

void aha_oracle_decode_step(const double *q, const double *k_new, const double *v_new,
                            int64_t problems, int64_t G, int64_t d,
                            int64_t budget, int64_t recent, int64_t slots,
                            int64_t logical_pos,
                            int scale_mode, double fixed_scale, double lambda_floor,
                            double *Kc, double *Vc, double *Fc, int32_t *pos,
                            int32_t *free_slot, double *out)
{
    aha_oracle_decode_step_ext(q, k_new, v_new, problems, G, d, budget, recent, slots,
                               logical_pos, scale_mode, fixed_scale, lambda_floor, 0, 0,
                               Kc, Vc, Fc, pos, free_slot, out);
}

/* ------------------------------------------------------------------------
 * The generation step with two options that the paper names without fixing
 * them for generation:
 *   sink          tokens at positions < sink are never evicted (the static
 *                 policy of the related work: the beginning tokens are kept);
 *   value_prior   the probabilities added to the running scores are refined
 *                 by the value prior (Sec. 4.3) inside the generation loop too.
 * READING for value_prior: nu_s = ||Vc[s]||^2 over the budget + 1 live slots
 * (the new token included), gamma_bar_s = nu_s / max over the live slots, no
 * average pool (neighbouring slots of the compact cache are not neighbouring
 * tokens); F[s] += gamma_bar_s * sum over the group's heads of the score
 * probabilities.  If every live value row is zero, gamma_bar = 1.
 * With sink = 0 and value_prior = 0 this is the step as the algorithm prints it.
 * ---------------------------------------------------------------------- */
void aha_oracle_decode_step_ext(const double *q, const double *k_new, const double *v_new,
                                int64_t problems, int64_t G, int64_t d,
                                int64_t budget, int64_t recent, int64_t slots,
                                int64_t logical_pos,
                                int scale_mode, double fixed_scale, double lambda_floor,
                                int64_t sink, int value_prior,
                                double *Kc, double *Vc, double *Fc, int32_t *pos,
                                int32_t *free_slot, double *out)
{
    int64_t live = budget + 1;
    double s_out = 1.0 / sqrt((double)d);
    double s_score = row_scale(scale_mode, fixed_scale, lambda_floor, logical_pos, budget, d);
#pragma omp parallel for schedule(dynamic)
    for (int64_t pr = 0; pr < problems; ++pr) {
        double *kc = Kc + pr * slots * d;
        double *vc = Vc + pr * slots * d;
        double *F = Fc + pr * slots;
        int32_t *ps = pos + pr * slots;
        int64_t fs = free_slot[pr];
        memcpy(kc + fs * d, k_new + pr * d, sizeof(double) * (size_t)d);
        memcpy(vc + fs * d, v_new + pr * d, sizeof(double) * (size_t)d);
        F[fs] = 0.0;
        ps[fs] = (int32_t)(logical_pos - 1);

        double *po = (double *)malloc(sizeof(double) * (size_t)live);
        double *pscore = (double *)malloc(sizeof(double) * (size_t)live);
        double *gbar = (double *)malloc(sizeof(double) * (size_t)live);
        for (int64_t s = 0; s < live; ++s) gbar[s] = 1.0;
        if (value_prior) {
            double numax = 0.0;
            for (int64_t s = 0; s < live; ++s) {
                double nu = 0.0;
                for (int64_t t = 0; t < d; ++t) nu += vc[s * d + t] * vc[s * d + t];
                gbar[s] = nu;
                if (nu > numax) numax = nu;
            }
            for (int64_t s = 0; s < live; ++s) gbar[s] = numax > 0.0 ? gbar[s] / numax : 1.0;
        }
        for (int64_t g = 0; g < G; ++g) {
            const double *qg = q + (pr * G + g) * d;
            softmax_row(qg, kc, live, d, s_out, po);
            softmax_row(qg, kc, live, d, s_score, pscore);
            double *o = out + (pr * G + g) * d;
            for (int64_t t = 0; t < d; ++t) o[t] = 0.0;
            for (int64_t s = 0; s < live; ++s)
                for (int64_t t = 0; t < d; ++t) o[t] += po[s] * vc[s * d + t];
            for (int64_t s = 0; s < live; ++s) F[s] += gbar[s] * pscore[s];
        }
        free(po);
        free(pscore);
        free(gbar);

        /* protected = the `recent` largest positions: positions are distinct,
         * so count how many live slots have a larger position */
        int64_t victim = -1;
        for (int64_t s = 0; s < live; ++s) {
            int64_t newer = 0;
            for (int64_t u = 0; u < live; ++u) if (ps[u] > ps[s]) ++newer;
            if (newer < recent) continue; /* protected: recent */
            if (ps[s] < sink) continue;   /* protected: sink token */
            if (victim < 0 || F[s] < F[victim] ||
                (F[s] == F[victim] && ps[s] > ps[victim]))
                victim = s;
        }
        ps[victim] = -1;
        free_slot[pr] = (int32_t)victim;
    }
}
