/*
 * PPOW window-scoring ORACLE -- test infrastructure, not product code.
 *
 * A plain, slow, double-precision CPU implementation of the per-window scoring
 * pass and the top-M window selection of PPOW ("Performance-Driven Policy
 * Optimization for Speculative Decoding with Adaptive Windowing").  Every
 * function is the paper's definition written out; there is no blocking, fusion
 * or reordering.  Only tests, the smoke check and the benchmark's cpu_baseline
 * leg may call it.  It shares no code, header, table or constant with the HIP
 * library: the codes below are the oracle's own.
 *
 * Storage types of a logit row: PPOW_ORACLE_F32 = IEEE binary32,
 * PPOW_ORACLE_BF16 = the upper 16 bits of a binary32 (uint16 storage).
 *
 * Pinned by tests/test_oracle_*.py against: the Cost-Aware Speedup Reward
 * column of Table 6, closed forms (V=2 Bernoulli entropy / KL, uniform and
 * one-hot targets), the identities of Appendix B.1 (sum of min = 1 - TV,
 * Pinsker), brute-force enumeration on tiny vocabularies, shift invariance and
 * float64 library routines (torch.log_softmax, scipy.special.rel_entr).
 * Parity unpinned: the proximity gap's first term when the caller supplies no
 * reference log-probability (Section 4.3.2 needs the target-greedy path, which
 * paired logits along the drafted path do not contain; the same-context
 * surrogate documented at ppow_oracle_score_windows is a reading, pinned only
 * to its own lse-free identity and to the K=1 case where both coincide).
 */
#ifndef PPOW_ORACLE_H
#define PPOW_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { PPOW_ORACLE_F32 = 0, PPOW_ORACLE_BF16 = 1 };
enum { PPOW_ORACLE_REJECTION = 0, PPOW_ORACLE_GREEDY = 1 };

/* Widen one stored logit row of length V to double, exactly. */
void ppow_oracle_widen_row(const void *row, int64_t V, int dtype, double *out);

/* log sum_y exp(x_y): two plain passes (max, then sum).  Section 4.2: P_t and
 * Q_t are the softmax distributions of the target / drafter logits. */
double ppow_oracle_logsumexp(const double *x, int64_t V);

/* Smallest index attaining max_y x_y.  Section 4.3.2: y_t = argmax_y pi_target. */
int64_t ppow_oracle_argmax(const double *x, int64_t V);

/* Shannon entropy H(P) in nats, P = softmax(a), lse_a = logsumexp(a).
 * Section 4.2 (confidence factor). */
double ppow_oracle_entropy(const double *a, int64_t V, double lse_a);

/* D_KL(P || Q) in nats, P = softmax(a), Q = softmax(b).  Section 4.2. */
double ppow_oracle_kl(const double *a, const double *b, int64_t V,
                      double lse_a, double lse_b);

/* C(P) = 1 - H(P) / log|V|.  Section 4.2, Appendix B.2. */
double ppow_oracle_confidence(double entropy, int64_t V);

/* Expected acceptance probability sum_y min(P(y), Q(y)).  Appendix B.1. */
double ppow_oracle_expected_accept(const double *a, const double *b, int64_t V,
                                   double lse_a, double lse_b);

/* Total variation distance (1/2) sum_y |P(y) - Q(y)|.  Appendix B.1. */
double ppow_oracle_total_variation(const double *a, const double *b, int64_t V,
                                   double lse_a, double lse_b);

/* alpha = min(1, P(tok) / Q(tok)) from the two log-probabilities.
 * Appendix C.1 (rejection-sampling verification). */
double ppow_oracle_accept_prob(double logp_target_tok, double logp_draft_tok);

/* tau = sum_{n=1..K} prod_{t=1..n} accept_t.  Appendix C.1. */
int32_t ppow_oracle_accepted_length(const int32_t *accept, int32_t K);

/* R_speedup = k / (k * gamma + 1).  Section 4.3.1. */
double ppow_oracle_speedup_reward(int32_t k, double gamma);

/* eta * 1[k == 0] * 1[delta < eps].  Section 4.3.2 with the k = 0 gate of
 * Algorithm 1's reward line. */
double ppow_oracle_proximity_reward(int32_t k, double delta, double eps, double eta);

/* Alignment divergence exp(d) - d - 1, d = log P(tok) - log Q(tok).  Appendix E. */
double ppow_oracle_alignment_metric(double logp_target_tok, double logp_draft_tok);

/* Group-relative advantage (R_i - mean) / (std + delta_stab) over one rollout
 * group of G rewards; std is the population standard deviation.  Section 4.1. */
void ppow_oracle_group_advantage(const double *rewards, int32_t G, double delta_stab,
                                 double *advantage);

/*
 * Score B windows of K drafted positions over a vocabulary of V.
 *
 * Inputs (host memory, caller-owned, dense row-major):
 *   draft_logits, target_logits  [B, K, V]  in `dtype` storage
 *   draft_tokens                 [B, K]     int32, 0 <= tok < V
 *   uniforms                     [B, K]     double; may be NULL in greedy mode
 *   ref_logprob                  [B] double or NULL.  When given it is the
 *       cumulative target log-probability of the target-preferred reference
 *       window (first term of the proximity gap, Section 4.3.2).  When NULL the
 *       reference token at each position is the argmax of the SAME target row
 *       that scores the drafted token ("same base context" reading): the gap
 *       becomes sum_t [log P_t(argmax) - log P_t(drafted)].
 *   verify: PPOW_ORACLE_REJECTION -> accept_t = [u_t <= alpha_t]  (Appendix C.1)
 *           PPOW_ORACLE_GREEDY    -> accept_t = [drafted_t == argmax_y P_t(y)]
 *
 * Outputs (any may be NULL):
 *   per window [B]: accepted_len (int32), r_speedup, r_proximity, adaw_score,
 *                   delta
 *   per position [B*K]: kl, confidence, entropy, accept_prob, expected_accept,
 *                   reverse_kl (D_KL(Q || P), the target-anchored regulariser of
 *                   Section 4.1 / Appendix A.2), logp_target_tok, logp_draft_tok,
 *                   alignment (Appendix E), argmax_target (int64)
 *
 * adaw_score = (1/K) sum_t C(P_t) * KL(P_t || Q_t) over all K positions.
 * Windows are scored by an OpenMP loop over b when built with -fopenmp;
 * `threads_used` (may be NULL) receives the thread count.  Returns 0, or
 * -1 on an invalid argument.
 */
typedef struct {
    int32_t *accepted_len;
    double *r_speedup, *r_proximity, *adaw_score, *delta;
    double *kl, *confidence, *entropy, *accept_prob, *expected_accept;
    double *reverse_kl, *logp_target_tok, *logp_draft_tok, *alignment;
    int64_t *argmax_target;
} ppow_oracle_outputs;

int ppow_oracle_score_windows(const void *draft_logits, const void *target_logits,
                              const int32_t *draft_tokens, const double *uniforms,
                              const double *ref_logprob,
                              int64_t B, int32_t K, int64_t V, int dtype,
                              double gamma, double eps, double eta, int verify,
                              const ppow_oracle_outputs *out, int32_t *threads_used);

/* Best candidate of each group of G consecutive windows (multi-candidate speculative
 * decoding: the candidate with the longest accepted prefix is the one that is kept;
 * Section 4.1, Table 2): best_len[g] = max accepted length in group g, best_index[g] =
 * index within the group of the first window attaining it.  Returns 0, or -1 on an invalid
 * argument (G < 1, B not a multiple of G). */
int ppow_oracle_group_best(const int32_t *accepted_len, int64_t B, int32_t G,
                           int32_t *best_len, int32_t *best_index);

/*
 * Sequence-mode ADAW (Algorithm 1, "Compute criticality score" and "ADAW-based window
 * selection"): for N sequences of T teacher-forced positions,
 *   criticality[n, t]  = C(P_t) * KL(P_t || Q_t)                       t = 0..T-1
 *   window_score[n, j] = (1/K) * sum_{t=j}^{j+K-1} criticality[n, t]   j = 0..T-K
 * Logits are [N, T, V] in `dtype` storage.  Outputs may be NULL.  Returns 0 or -1.
 */
int ppow_oracle_adaw_sequence(const void *draft_logits, const void *target_logits,
                              int64_t N, int32_t T, int64_t V, int dtype, int32_t K,
                              double *criticality, double *window_score);

/*
 * Sample one window start per sequence from weights proportional to the window scores
 * (Algorithm 1), by inverting the cumulative distribution with the given uniform draw u in
 * [0,1): with c_j = sum_{i<=j} s_i, the start is the smallest j with c_j >= u * c_{W-1}
 * (the last j if rounding leaves none).  If every score of a sequence is zero the weights
 * are undefined and the start is drawn uniformly: floor(u * W), capped at W-1.
 * score is [N, W]; returns 0 or -1.
 */
int ppow_oracle_sample_starts(const double *score, int64_t N, int64_t W, const double *uniforms,
                              int64_t *start);

/*
 * Window starts under the hard-window curriculum (Appendix A.3, Table 5: the proportion of
 * ADAW-selected windows grows 0.2 / 0.4 / 0.6 over training): sequence n gets an ADAW-selected
 * start -- ppow_oracle_sample_starts with uniforms[n] -- when mix_uniforms[n] < adaw_fraction,
 * and otherwise an ordinary window, every start equally likely: floor(uniforms[n] * W), capped
 * at W-1.  (The paper does not say how the remaining windows are chosen; uniform starts are
 * this build's reading.)  adaw_fraction in [0, 1]; returns 0 or -1.
 */
int ppow_oracle_sample_starts_curriculum(const double *score, int64_t N, int64_t W,
                                         const double *uniforms, const double *mix_uniforms,
                                         double adaw_fraction, int64_t *start);

/*
 * Top-M selection: the M windows with the largest score, ordered by score
 * descending and, among equal scores, by index ascending (a full stable sort,
 * first M kept).  Section 4.2: windows with larger s_j are prioritised.
 * Returns 0, or -1 on an invalid argument (M < 1, M > B, NULL).
 */
int ppow_oracle_select_windows(const double *score, int64_t B, int64_t M,
                               int64_t *indices);

#ifdef __cplusplus
}
#endif
#endif
