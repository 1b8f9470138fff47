/*
 * PPOW window-scoring ORACLE -- test infrastructure, not product code.
 * See ppow_oracle.h for the contract, the pins and what is unpinned.
 *
 * Everything is computed in double from the exactly widened stored logits,
 * with the definitions of the paper written out one after the other.
 */
#include "ppow_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

void ppow_oracle_widen_row(const void *row, int64_t V, int dtype, double *out)
{
    if (dtype == PPOW_ORACLE_BF16) {
        const uint16_t *h = (const uint16_t *)row;
        for (int64_t y = 0; y < V; ++y) {
            /* a bfloat16 is the upper half of a binary32 */
            uint32_t bits = (uint32_t)h[y] << 16;
            float f;
            memcpy(&f, &bits, sizeof f);
            out[y] = (double)f;
        }
    } else {
        const float *f = (const float *)row;
        for (int64_t y = 0; y < V; ++y) out[y] = (double)f[y];
    }
}

double ppow_oracle_logsumexp(const double *x, int64_t V)
{
    double m = x[0];
    for (int64_t y = 1; y < V; ++y)
        if (x[y] > m) m = x[y];
    double z = 0.0;
    for (int64_t y = 0; y < V; ++y) z += exp(x[y] - m);
    return m + log(z);
}

int64_t ppow_oracle_argmax(const double *x, int64_t V)
{
    int64_t best = 0;
    for (int64_t y = 1; y < V; ++y)
        if (x[y] > x[best]) best = y; /* strict: the smallest index wins ties */
    return best;
}

double ppow_oracle_entropy(const double *a, int64_t V, double lse_a)
{
    double h = 0.0;
    for (int64_t y = 0; y < V; ++y) {
        double logp = a[y] - lse_a;
        double p = exp(logp);
        if (p > 0.0) h -= p * logp; /* 0 log 0 = 0 */
    }
    return h;
}

double ppow_oracle_kl(const double *a, const double *b, int64_t V,
                      double lse_a, double lse_b)
{
    double kl = 0.0;
    for (int64_t y = 0; y < V; ++y) {
        double logp = a[y] - lse_a;
        double logq = b[y] - lse_b;
        double p = exp(logp);
        if (p > 0.0) kl += p * (logp - logq);
    }
    return kl;
}

double ppow_oracle_confidence(double entropy, int64_t V)
{
    return 1.0 - entropy / log((double)V);
}

double ppow_oracle_expected_accept(const double *a, const double *b, int64_t V,
                                   double lse_a, double lse_b)
{
    double s = 0.0;
    for (int64_t y = 0; y < V; ++y) {
        double p = exp(a[y] - lse_a);
        double q = exp(b[y] - lse_b);
        s += (p < q) ? p : q;
    }
    return s;
}

double ppow_oracle_total_variation(const double *a, const double *b, int64_t V,
                                   double lse_a, double lse_b)
{
    double s = 0.0;
    for (int64_t y = 0; y < V; ++y) {
        double p = exp(a[y] - lse_a);
        double q = exp(b[y] - lse_b);
        s += fabs(p - q);
    }
    return 0.5 * s;
}

double ppow_oracle_accept_prob(double logp_target_tok, double logp_draft_tok)
{
    /* min(1, P/Q) taken in the log domain so that Q -> 0 cannot divide by 0 */
    double log_ratio = logp_target_tok - logp_draft_tok;
    return (log_ratio >= 0.0) ? 1.0 : exp(log_ratio);
}

int32_t ppow_oracle_accepted_length(const int32_t *accept, int32_t K)
{
    int32_t tau = 0;
    for (int32_t n = 1; n <= K; ++n) {
        int32_t prod = 1;
        for (int32_t t = 1; t <= n; ++t) prod *= (accept[t - 1] != 0);
        tau += prod;
    }
    return tau;
}

double ppow_oracle_speedup_reward(int32_t k, double gamma)
{
    return (double)k / ((double)k * gamma + 1.0);
}

double ppow_oracle_proximity_reward(int32_t k, double delta, double eps, double eta)
{
    return (k == 0 && delta < eps) ? eta : 0.0;
}

double ppow_oracle_alignment_metric(double logp_target_tok, double logp_draft_tok)
{
    double d = logp_target_tok - logp_draft_tok;
    return exp(d) - d - 1.0;
}

void ppow_oracle_group_advantage(const double *rewards, int32_t G, double delta_stab,
                                 double *advantage)
{
    double mu = 0.0;
    for (int32_t i = 0; i < G; ++i) mu += rewards[i];
    mu /= (double)G;
    double var = 0.0;
    for (int32_t i = 0; i < G; ++i) var += (rewards[i] - mu) * (rewards[i] - mu);
    double sigma = sqrt(var / (double)G);
    for (int32_t i = 0; i < G; ++i) advantage[i] = (rewards[i] - mu) / (sigma + delta_stab);
}

static void score_one_window(const void *draft_logits, const void *target_logits,
                             const int32_t *draft_tokens, const double *uniforms,
                             const double *ref_logprob, int64_t b, int32_t K, int64_t V,
                             int dtype, double gamma, double eps, double eta, int verify,
                             const ppow_oracle_outputs *out, double *a, double *q_row,
                             int32_t *accept)
{
    const size_t esz = (dtype == PPOW_ORACLE_BF16) ? 2 : 4;
    double sum_v = 0.0;          /* sum_t C(P_t) KL(P_t || Q_t) */
    double sum_ref = 0.0;        /* sum_t log P_t(reference token) */
    double sum_drafted = 0.0;    /* sum_t log P_t(drafted token)   */

    for (int32_t t = 0; t < K; ++t) {
        const int64_t row = b * (int64_t)K + t;
        const char *ta = (const char *)target_logits + (size_t)row * (size_t)V * esz;
        const char *db = (const char *)draft_logits + (size_t)row * (size_t)V * esz;
        ppow_oracle_widen_row(ta, V, dtype, a);
        ppow_oracle_widen_row(db, V, dtype, q_row);

        const double lse_a = ppow_oracle_logsumexp(a, V);
        const double lse_b = ppow_oracle_logsumexp(q_row, V);
        const double H = ppow_oracle_entropy(a, V, lse_a);
        const double kl = ppow_oracle_kl(a, q_row, V, lse_a, lse_b);
        const double C = ppow_oracle_confidence(H, V);
        const int64_t ystar = ppow_oracle_argmax(a, V);
        const int64_t tok = draft_tokens[row];
        const double logp_tok = a[tok] - lse_a;
        const double logq_tok = q_row[tok] - lse_b;
        const double alpha = ppow_oracle_accept_prob(logp_tok, logq_tok);

        if (verify == PPOW_ORACLE_GREEDY)
            accept[t] = (tok == ystar);
        else
            accept[t] = (uniforms[row] <= alpha);

        sum_v += C * kl;
        sum_ref += a[ystar] - lse_a;
        sum_drafted += logp_tok;

        if (out->kl) out->kl[row] = kl;
        if (out->confidence) out->confidence[row] = C;
        if (out->entropy) out->entropy[row] = H;
        if (out->accept_prob) out->accept_prob[row] = alpha;
        if (out->expected_accept)
            out->expected_accept[row] = ppow_oracle_expected_accept(a, q_row, V, lse_a, lse_b);
        if (out->reverse_kl) out->reverse_kl[row] = ppow_oracle_kl(q_row, a, V, lse_b, lse_a);
        if (out->logp_target_tok) out->logp_target_tok[row] = logp_tok;
        if (out->logp_draft_tok) out->logp_draft_tok[row] = logq_tok;
        if (out->alignment) out->alignment[row] = ppow_oracle_alignment_metric(logp_tok, logq_tok);
        if (out->argmax_target) out->argmax_target[row] = ystar;
    }

    const int32_t k = ppow_oracle_accepted_length(accept, K);
    const double first_term = ref_logprob ? ref_logprob[b] : sum_ref;
    const double delta = first_term - sum_drafted;

    if (out->accepted_len) out->accepted_len[b] = k;
    if (out->r_speedup) out->r_speedup[b] = ppow_oracle_speedup_reward(k, gamma);
    if (out->r_proximity) out->r_proximity[b] = ppow_oracle_proximity_reward(k, delta, eps, eta);
    if (out->adaw_score) out->adaw_score[b] = sum_v / (double)K;
    if (out->delta) out->delta[b] = delta;
}

int ppow_oracle_score_windows(const void *draft_logits, const void *target_logits,
                              const int32_t *draft_tokens, const double *uniforms,
                              const double *ref_logprob,
                              int64_t B, int32_t K, int64_t V, int dtype,
                              double gamma, double eps, double eta, int verify,
                              const ppow_oracle_outputs *out, int32_t *threads_used)
{
    if (!draft_logits || !target_logits || !draft_tokens || !out) return -1;
    if (B < 0 || K < 1 || V < 2) return -1;
    if (dtype != PPOW_ORACLE_F32 && dtype != PPOW_ORACLE_BF16) return -1;
    if (verify != PPOW_ORACLE_REJECTION && verify != PPOW_ORACLE_GREEDY) return -1;
    if (verify == PPOW_ORACLE_REJECTION && !uniforms) return -1;
    for (int64_t i = 0; i < B * (int64_t)K; ++i)
        if (draft_tokens[i] < 0 || draft_tokens[i] >= V) return -1;

    int32_t nthreads = 1;
    int failed = 0;
#ifdef _OPENMP
#pragma omp parallel
#endif
    {
#ifdef _OPENMP
#pragma omp single
        nthreads = omp_get_num_threads();
#endif
        double *a = (double *)malloc((size_t)V * sizeof(double));
        double *q_row = (double *)malloc((size_t)V * sizeof(double));
        int32_t *accept = (int32_t *)malloc((size_t)K * sizeof(int32_t));
        if (!a || !q_row || !accept) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
            failed = 1;
        }
#ifdef _OPENMP
#pragma omp barrier
#pragma omp for schedule(dynamic, 1)
#endif
        for (int64_t b = 0; b < B; ++b) {
            if (!failed)
                score_one_window(draft_logits, target_logits, draft_tokens, uniforms,
                                 ref_logprob, b, K, V, dtype, gamma, eps, eta, verify, out,
                                 a, q_row, accept);
        }
        free(a);
        free(q_row);
        free(accept);
    }
    if (threads_used) *threads_used = nthreads;
    return failed ? -1 : 0;
}

int ppow_oracle_group_best(const int32_t *accepted_len, int64_t B, int32_t G,
                           int32_t *best_len, int32_t *best_index)
{
    if (!accepted_len || !best_len || !best_index || G < 1 || B < 0 || B % G != 0) return -1;
    for (int64_t g = 0; g < B / G; ++g) {
        int32_t best = 0;
        for (int32_t i = 1; i < G; ++i)
            if (accepted_len[g * G + i] > accepted_len[g * G + best]) best = i;   /* first maximum */
        best_len[g] = accepted_len[g * G + best];
        best_index[g] = best;
    }
    return 0;
}

int ppow_oracle_adaw_sequence(const void *draft_logits, const void *target_logits,
                              int64_t N, int32_t T, int64_t V, int dtype, int32_t K,
                              double *criticality, double *window_score)
{
    if (!draft_logits || !target_logits || N < 0 || T < 1 || K < 1 || K > T || V < 2) return -1;
    if (dtype != PPOW_ORACLE_F32 && dtype != PPOW_ORACLE_BF16) return -1;
    const size_t esz = (dtype == PPOW_ORACLE_BF16) ? 2 : 4;
    const int64_t W = (int64_t)T - K + 1;
    int failed = 0;
#ifdef _OPENMP
#pragma omp parallel
#endif
    {
        double *a = (double *)malloc((size_t)V * sizeof(double));
        double *b = (double *)malloc((size_t)V * sizeof(double));
        double *v = (double *)malloc((size_t)T * sizeof(double));
        if (!a || !b || !v) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
            failed = 1;
        }
#ifdef _OPENMP
#pragma omp barrier
#pragma omp for schedule(dynamic, 1)
#endif
        for (int64_t n = 0; n < N; ++n) {
            if (failed) continue;
            for (int32_t t = 0; t < T; ++t) {
                const int64_t row = n * (int64_t)T + t;
                ppow_oracle_widen_row((const char *)target_logits + (size_t)row * (size_t)V * esz, V, dtype, a);
                ppow_oracle_widen_row((const char *)draft_logits + (size_t)row * (size_t)V * esz, V, dtype, b);
                const double lse_a = ppow_oracle_logsumexp(a, V);
                const double lse_b = ppow_oracle_logsumexp(b, V);
                const double H = ppow_oracle_entropy(a, V, lse_a);
                v[t] = ppow_oracle_confidence(H, V) * ppow_oracle_kl(a, b, V, lse_a, lse_b);
                if (criticality) criticality[row] = v[t];
            }
            if (window_score) {
                for (int64_t j = 0; j < W; ++j) {
                    double sum = 0.0;
                    for (int32_t t = 0; t < K; ++t) sum += v[j + t];
                    window_score[n * W + j] = sum / (double)K;
                }
            }
        }
        free(a);
        free(b);
        free(v);
    }
    return failed ? -1 : 0;
}

int ppow_oracle_sample_starts(const double *score, int64_t N, int64_t W, const double *uniforms,
                              int64_t *start)
{
    if (!score || !uniforms || !start || N < 0 || W < 1) return -1;
    for (int64_t n = 0; n < N; ++n) {
        const double *s = score + n * W;
        double total = 0.0;
        for (int64_t j = 0; j < W; ++j) total += s[j];
        const double u = uniforms[n];
        if (!(total > 0.0)) {
            int64_t j = (int64_t)floor(u * (double)W);
            start[n] = j < W - 1 ? j : W - 1;
            continue;
        }
        const double threshold = u * total;
        double c = 0.0;
        int64_t pick = W - 1;
        for (int64_t j = 0; j < W; ++j) {
            c += s[j];
            if (c >= threshold) { pick = j; break; }
        }
        start[n] = pick;
    }
    return 0;
}

int ppow_oracle_sample_starts_curriculum(const double *score, int64_t N, int64_t W,
                                         const double *uniforms, const double *mix_uniforms,
                                         double adaw_fraction, int64_t *start)
{
    if (!score || !uniforms || !mix_uniforms || !start || N < 0 || W < 1) return -1;
    if (!(adaw_fraction >= 0.0 && adaw_fraction <= 1.0)) return -1;
    for (int64_t n = 0; n < N; ++n) {
        if (mix_uniforms[n] < adaw_fraction) {
            /* an ADAW-selected window: proportional to the window scores */
            if (ppow_oracle_sample_starts(score + n * W, 1, W, uniforms + n, start + n) != 0)
                return -1;
        } else {
            /* an ordinary window: every start equally likely */
            int64_t j = (int64_t)floor(uniforms[n] * (double)W);
            start[n] = j < W - 1 ? j : W - 1;
        }
    }
    return 0;
}

typedef struct {
    double score;
    int64_t index;
} scored_window;

static int by_score_desc_then_index(const void *lhs, const void *rhs)
{
    const scored_window *l = (const scored_window *)lhs;
    const scored_window *r = (const scored_window *)rhs;
    if (l->score > r->score) return -1;
    if (l->score < r->score) return 1;
    return (l->index > r->index) - (l->index < r->index);
}

int ppow_oracle_select_windows(const double *score, int64_t B, int64_t M, int64_t *indices)
{
    if (!score || !indices || M < 1 || M > B) return -1;
    scored_window *w = (scored_window *)malloc((size_t)B * sizeof(scored_window));
    if (!w) return -1;
    for (int64_t i = 0; i < B; ++i) {
        w[i].score = score[i];
        w[i].index = i;
    }
    /* the index is part of the key, so any comparison sort gives the stable order */
    qsort(w, (size_t)B, sizeof(scored_window), by_score_desc_then_index);
    for (int64_t i = 0; i < M; ++i) indices[i] = w[i].index;
    free(w);
    return 0;
}
