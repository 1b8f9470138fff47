/*
 * libppow -- window-level scoring pass of PPOW drafter optimisation on AMD MI355X
 * (gfx950), as a C-ABI library.
 *
 * For B speculative windows of K drafted tokens it streams the paired drafter
 * and target logit rows once and returns, per window, the verification outcome
 * (accepted prefix length), the Cost-Aware Speedup Reward, the Distribution-Based
 * Proximity Reward and the ADAW priority score; a second entry point selects the
 * M windows of largest score.  All data pointers are DEVICE pointers owned by
 * the caller; the library neither allocates, frees nor keeps them.  The params /
 * outputs structs are HOST structs read during the call.  Calls enqueue work on
 * `hip_stream` (a hipStream_t cast to void*; NULL = the default stream) and
 * return without synchronising: outputs are valid once the stream has drained.
 * Results are deterministic run to run (no floating-point atomics).
 *
 * Every entry point returns a ppow_status.  Errors that the host can see are
 * reported before anything is launched; ppow_last_error() then holds a message.
 */
#ifndef PPOW_H
#define PPOW_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PPOW_OK = 0,
    PPOW_ERR_INVALID_ARG = 1,  /* NULL required pointer, size or enum out of range */
    PPOW_ERR_UNSUPPORTED = 2,  /* valid request outside a built-in limit (the rows
                                  ppow_score_windows_static holds)                 */
    PPOW_ERR_WORKSPACE = 3,    /* workspace NULL, misaligned or too small          */
    PPOW_ERR_DEVICE = 4        /* a HIP launch reported an error                   */
} ppow_status;

/* Storage type of both logit tensors. */
typedef enum { PPOW_F32 = 0, PPOW_BF16 = 1 } ppow_dtype;

/* Verification rule.  REJECTION: position t is accepted iff u_t <= alpha_t with
 * alpha_t = min(1, P_t(tok)/Q_t(tok)) (Appendix C.1).  GREEDY: accepted iff the
 * drafted token is the target's argmax, the temperature-0 limit of the same rule
 * (Table 5 lists temperature 0.0 among the decoding settings). */
typedef enum { PPOW_VERIFY_REJECTION = 0, PPOW_VERIFY_GREEDY = 1 } ppow_verify;

enum {
    /* also compute sum_y min(P_t(y), Q_t(y)), the expected acceptance probability
     * of Appendix B.1; it needs normalised probabilities, hence a second pass over
     * each row pair, served from registers and LDS (a cluster of workgroups shares
     * a row pair, every logit is fetched from memory once) where the sizes allow
     * it, from memory otherwise -- also while the stream is being captured into a
     * graph.  Calls with this flag on different streams of one device run one
     * after another (each such kernel needs the whole device); the library orders
     * them with one event per device, see ppow_release() */
    PPOW_FLAG_EXPECTED_ACCEPT = 1u,
    /* also compute the forward values of the policy-loss terms from the same pass:
     * KL(Q_t || P_t), the target-anchored regulariser of Section 4.1 / Appendix A.2,
     * and the alignment metric exp(d) - d - 1, d = log P_t(tok) - log Q_t(tok), of
     * Appendix E; one more multiply-add per logit pair */
    PPOW_FLAG_POLICY_TERMS = 2u
};

#define PPOW_MAX_K 64          /* drafted positions per window (one wavefront) */

typedef struct {
    float cost_ratio;  /* gamma > 0: drafter cost relative to the target (Section 4.3.1) */
    float prox_eps;    /* epsilon: proximity tolerance, Table 5 default 0.5             */
    float prox_eta;    /* eta: proximity reward scale, Table 5 default 1.0              */
    int32_t verify;    /* ppow_verify                                                   */
    uint32_t flags;    /* PPOW_FLAG_*                                                   */
    int32_t rollout_group; /* G: windows per rollout group for `advantage` (Table 5: 8);
                              0 when the advantage output is not used; must divide B    */
    float adv_delta;   /* small positive constant in the advantage normalisation        */
} ppow_params;

/* Device output arrays.  The first four are required; the rest may be NULL. */
typedef struct {
    int32_t *accepted_len;   /* [B]   k: accepted prefix length, 0..K (Appendix C.1)          */
    float *r_speedup;        /* [B]   k / (k*gamma + 1)              (Section 4.3.1)          */
    float *r_proximity;      /* [B]   eta * [k == 0] * [delta < eps] (Section 4.3.2, Alg. 1)  */
    float *adaw_score;       /* [B]   (1/K) sum_t C(P_t) KL(P_t||Q_t) (Section 4.2)           */
    float *delta;            /* [B]   proximity gap                  (Section 4.3.2)          */
    float *kl;               /* [B*K] KL(P_t || Q_t) in nats                                  */
    float *confidence;       /* [B*K] C(P_t) = 1 - H(P_t)/ln V                                */
    float *accept_prob;      /* [B*K] alpha_t                                                 */
    float *expected_accept;  /* [B*K] sum_y min(P_t, Q_t); needs PPOW_FLAG_EXPECTED_ACCEPT    */
    float *logp_target_tok;  /* [B*K] log P_t(drafted token)                                  */
    float *logp_draft_tok;   /* [B*K] log Q_t(drafted token)                                  */
    float *reverse_kl;       /* [B*K] KL(Q_t || P_t); needs PPOW_FLAG_POLICY_TERMS            */
    float *alignment;        /* [B*K] exp(d) - d - 1 (Appendix E); needs PPOW_FLAG_POLICY_TERMS */
    float *reverse_kl_mean;  /* [B]   mean over the window's K positions; same flag           */
    float *alignment_mean;   /* [B]   mean over the window's K positions; same flag           */
    float *advantage;        /* [B]   group-relative advantage (R_i - mean)/(std + delta) of
                                      R_i = r_speedup + r_proximity over groups of
                                      rollout_group consecutive windows (Section 4.1);
                                      population standard deviation; needs rollout_group >= 1 */
    int32_t *group_best_len; /* [B/G] largest accepted length among the G = rollout_group
                                      candidate windows of a group (multi-candidate decoding,
                                      Table 2)                                                 */
    int32_t *group_best_index;/* [B/G] index within the group of the first window attaining it */
} ppow_outputs;

/* Bytes of device workspace ppow_score_windows needs for these sizes (0 on
 * invalid sizes).  The workspace must be 16-byte aligned.  After the stream has
 * drained, the first 32-bit word of the workspace is 0 unless the bounded wait
 * inside the cluster variant of the row kernel expired, which is not expected to
 * happen; every window of that call is then reported with accepted_len = -3,
 * zero rewards and adaw_score = 0 (its other outputs are unspecified). */
size_t ppow_score_workspace_bytes(int64_t B, int32_t K, int64_t V, int32_t dtype, uint32_t flags);

/*
 * Score B windows (Algorithm 1: criticality and window score, Verify, proximity
 * gap and reward lines).
 *
 *   draft_logits, target_logits  [B, K, V] dense row-major, V contiguous, `dtype`
 *                                storage, base pointers 16-byte aligned.  Logits
 *                                must be finite; a window with a NaN or an
 *                                infinity in any of its rows is reported with
 *                                accepted_len = -2, zero rewards and adaw_score = 0
 *                                (its other outputs are unspecified).
 *                                P_t = softmax(target row), Q_t = softmax(draft
 *                                row), temperature 1.
 *   draft_tokens                 [B, K] int32, 0 <= token < V.  The host cannot
 *                                see them, so the device checks: a token outside
 *                                the range is never used as an address; its
 *                                window gets accepted_len = -1, r_speedup = 0 and
 *                                r_proximity = 0 (adaw_score, kl, confidence and
 *                                expected_accept do not depend on the tokens and
 *                                stay valid; the token-dependent per-position
 *                                outputs of that window are unspecified).
 *   uniforms                     [B, K] float32 draws u_t in [0,1]; may be NULL
 *                                only for PPOW_VERIFY_GREEDY
 *   ref_logprob                  [B] float32 or NULL.  When given it is the
 *                                cumulative target log-probability of the
 *                                target-preferred reference window, the first
 *                                term of the proximity gap of Section 4.3.2.
 *                                When NULL the reference token of position t is
 *                                the argmax of the same target row, so that
 *                                delta = sum_t (max_y a_t[y] - a_t[tok_t]).
 *   B >= 0 (B = 0 is a no-op), 1 <= K <= PPOW_MAX_K, 2 <= V < 2^31.
 *
 * The ADAW score averages over all K positions whether or not verification
 * stopped earlier.  r_proximity is the gated value that enters the window
 * reward; the caller adds r_speedup + r_proximity.
 */
int ppow_score_windows(const void *draft_logits, const void *target_logits,
                       const int32_t *draft_tokens, const float *uniforms,
                       const float *ref_logprob,
                       int64_t B, int32_t K, int64_t V, int32_t dtype,
                       const ppow_params *params, const ppow_outputs *out,
                       void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * ppow_score_windows for callers that cannot allocate device memory or carry a
 * workspace around: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same arguments, outputs, kernels and error behaviour as
 * ppow_score_windows, minus the workspace: the records between the row kernel
 * and the window epilogue live in an array built into the library
 * (PPOW_STATIC_SCRATCH_BYTES of device memory per GPU the library is used on,
 * held until the process ends).  B*K must not exceed PPOW_STATIC_MAX_ROWS
 * (PPOW_ERR_UNSUPPORTED otherwise: use ppow_score_windows).  The call allocates
 * and frees nothing; its first call on a device resolves the array's address
 * and creates the event described at ppow_release().  All calls on one GPU share
 * that GPU's array: calls that overlap in time on one GPU (two streams, two
 * threads) race and give undefined outputs -- order them yourself.
 */
#define PPOW_STATIC_MAX_ROWS 131072     /* B*K; 16384 windows of K = 8 */
#define PPOW_STATIC_SCRATCH_BYTES ((1u << 20) + 32u * PPOW_STATIC_MAX_ROWS)   /* 5 MiB */
int ppow_score_windows_static(const void *draft_logits, const void *target_logits,
                              const int32_t *draft_tokens, const float *uniforms,
                              const float *ref_logprob,
                              int64_t B, int32_t K, int64_t V, int32_t dtype,
                              const ppow_params *params, const ppow_outputs *out,
                              void *hip_stream);

/* Bytes of device workspace ppow_adaw_sequence needs (0 on invalid sizes). */
size_t ppow_adaw_sequence_workspace_bytes(int64_t N, int32_t T, int64_t V, int32_t dtype);

/*
 * Sequence-mode ADAW (Algorithm 1, criticality and window-selection lines): N sequences of
 * T teacher-forced positions are scored ONCE (each logit row is read once although every
 * position belongs to up to K overlapping windows), then
 *   criticality[n, t]  = C(P_t) * KL(P_t || Q_t)                         t = 0..T-1
 *   window_score[n, j] = (1/K) sum_{t=j}^{j+K-1} criticality[n, t]       j = 0..T-K
 * and, if asked, one window start per sequence.  Under the hard-window curriculum
 * (Appendix A.3, Table 5: the proportion of ADAW-selected windows grows 0.2 / 0.4 / 0.6 over
 * training) sequence n gets an ADAW-selected start when mix_uniforms[n] < adaw_fraction and
 * an ordinary one, floor(uniforms[n] * (T-K+1)), otherwise (how the other windows are chosen
 * the paper does not say: uniformly random is this library's reading).  An ADAW-selected start
 * is drawn with probability proportional to the window scores: the smallest j whose cumulative
 * score reaches uniforms[n] times the total (running sums in double; if all scores are zero,
 * floor(u * (T-K+1))).
 *
 *   draft_logits, target_logits  [N, T, V] as in ppow_score_windows
 *   uniforms       [N] float32 in [0,1), required iff sampled_start is given
 *   adaw_fraction  in [0, 1]; 1 = every start ADAW-selected (Algorithm 1 as printed)
 *   mix_uniforms   [N] float32 in [0,1), required iff sampled_start is given and
 *                  adaw_fraction < 1
 *   criticality    [N*T] out or NULL;  window_score [N*(T-K+1)] out, required
 *   sampled_start  [N] int32 out or NULL
 *   N >= 0, 1 <= K <= T, N*T < 2^31, 2 <= V < 2^31.
 * ppow_select_windows can then rank all N*(T-K+1) windows.
 */
int ppow_adaw_sequence(const void *draft_logits, const void *target_logits,
                       int64_t N, int32_t T, int64_t V, int32_t dtype, int32_t K,
                       const float *uniforms, float adaw_fraction, const float *mix_uniforms,
                       float *criticality, float *window_score, int32_t *sampled_start,
                       void *workspace, size_t workspace_bytes, void *hip_stream);

/* Bytes of device workspace ppow_select_windows needs (0 on invalid sizes). */
size_t ppow_select_workspace_bytes(int64_t B, int32_t M);

/*
 * Top-M window selection (Section 4.2: windows with larger score are
 * prioritised).  Writes the indices of the M largest scores ordered by score
 * descending, equal scores by index ascending.
 *
 *   adaw_score  [B] float32, finite
 *   indices     [M] int32 out
 *   scores      [M] float32 out or NULL: the selected scores in the same order
 *   1 <= M <= B < 2^31.
 */
int ppow_select_windows(const float *adaw_score, int64_t B, int32_t M,
                        int32_t *indices, float *scores,
                        void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Releases what the library holds besides caller memory: the HIP event (one per
 * device) with which it orders the calls that use the on-chip second pass.
 * Optional; typically called once before the process ends, with no other thread
 * inside a libppow call.  Work already enqueued is not affected, and a later
 * scoring call simply creates the event again.
 */
int ppow_release(void);

/* Testing aid: how many times a workgroup of the on-chip second pass looks for
 * its partners' results before it gives up (0 = the default, about 2^24).  A
 * tiny value makes the give-up path -- status word set, windows marked with
 * accepted_len = -3 -- reachable from a test; every kernel still ends normally. */
void ppow_debug_cluster_wait_limit(uint32_t looks);

/* Message of the calling thread's most recent failed call (static storage). */
const char *ppow_last_error(void);

/* Which streaming kernel the calling thread's most recent ppow_score_windows call
 * launched: "row" (one workgroup per row pair), "cluster" (a cluster of workgroups
 * per row pair, second pass from LDS) or "none".  Static storage. */
const char *ppow_last_row_kernel(void);

/* Library version, "major.minor.patch". */
const char *ppow_version(void);

#ifdef __cplusplus
}
#endif
#endif
